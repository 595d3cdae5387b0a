#!/usr/bin/env python3
"""Benchmark of the MultiWrite dispatch hot path on one MI355X.

A step is one pass of the whole path over one batch: plan -> pack -> unpack (index, expand), all
through the C ABI, inputs resident in HBM; batches follow each other as in a steady stream, and
the default schedule issues a whole step as one launch (mw_stream_step: packer and expander as one
stream of workgroups, the latency-bound plan and receive index of the next batch riding along;
see step()).  The headline workload is the DeepSeek-V3-shaped
dispatch (64 simulated ranks, 256 experts, top-8 with group-limited routing, 4096 tokens of
7168 bf16 on this rank; 64 peer receive regions).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|c0|c1|c2|c3|c3_hot|c4]
                  [--schedule auto|aligned|pipelined|one_stream|one_launch|free|single] [--no-cpu-baseline]

Without --workload the line is C1's (with the variants measured on its shape and the oracle timed
on the host cores) plus a `configs` object with a block per configuration -- C0 tiny, C1, C2 fp8,
C3 256-rank Zipf, C3_HOT (its skew stress point) and C4 AllGather -- each timed briefly in the same
process: step time, GB/s, % of the HBM peak, schedule, bytes saved, and the roofline of its dominant
launch from at least 24 bracketed launches (average and median).  --workload cN times one
configuration alone, in full.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
N_SETS = 3                      # rotating buffer sets (> 1 GB touched per step, MALL is 256 MB)
METRIC = "dispatch pack+unpack HBM GB/s (% of peak) + bytes saved vs unicast, 1 GPU"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class TimingEvent:
    """A HIP event with timing, created without the system-scope fence that torch's events end
    with when they are recorded (a cache write-back and invalidation nothing here needs): the
    pair around a launch then measures about 2 us less of its own making.  Same interface as
    the part of torch.cuda.Event the bench uses."""
    _hip = None

    def __init__(self, torch):
        import ctypes as C
        if TimingEvent._hip is None:
            TimingEvent._hip = C.CDLL("libamdhip64.so")
        self._C, self._torch = C, torch
        ev = C.c_void_p()
        if TimingEvent._hip.hipEventCreateWithFlags(C.byref(ev), C.c_uint(0x20000000)) != 0:
            raise OSError("hipEventCreateWithFlags failed")
        self._ev = ev

    @property
    def cuda_event(self):
        return self._ev.value

    def record(self, stream=None):
        st = self._torch.cuda.current_stream() if stream is None else stream
        if TimingEvent._hip.hipEventRecord(self._ev, self._C.c_void_p(st.cuda_stream)) != 0:
            raise RuntimeError("hipEventRecord failed")

    def elapsed_time(self, other):
        ms = self._C.c_float()
        if TimingEvent._hip.hipEventElapsedTime(self._C.byref(ms), self._ev, other._ev) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)


def new_events(torch, n):
    try:
        ev = [(TimingEvent(torch), TimingEvent(torch)) for _ in range(n)]
    except OSError:          # the HIP runtime library cannot be opened by name: torch's events
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for a, b in ev:          # (torch creates its handles on first record)
        a.record(); b.record()
    torch.cuda.synchronize()
    return ev


class DeviceEvent:
    """Cross-stream ordering between kernels of this one device: a HIP event created with
    hipEventDisableTiming | hipEventDisableSystemFence.  torch's events end with a
    system-scope fence (cache write-back and invalidation) when they are recorded, which nothing
    here needs -- no host code or other device reads what the kernels wrote -- and which costs
    about 2 us per step on the stream that records.  Falls back to a torch event if the HIP
    runtime library cannot be opened by name."""
    _hip = None

    def __init__(self, torch):
        import ctypes as C
        self._C, self._torch_ev, self._ev = C, None, None
        try:
            if DeviceEvent._hip is None:
                DeviceEvent._hip = C.CDLL("libamdhip64.so")
            ev = C.c_void_p()
            if DeviceEvent._hip.hipEventCreateWithFlags(C.byref(ev), C.c_uint(0x2 | 0x20000000)) != 0:
                raise OSError("hipEventCreateWithFlags failed")
            self._ev = ev
        except OSError:
            self._torch_ev = torch.cuda.Event()

    def record(self, stream):
        if self._ev is None:
            self._torch_ev.record(stream)
        elif DeviceEvent._hip.hipEventRecord(self._ev, self._C.c_void_p(stream.cuda_stream)) != 0:
            raise RuntimeError("hipEventRecord failed")

    def make_wait(self, stream):
        """`stream` waits for the work recorded so far."""
        if self._ev is None:
            stream.wait_event(self._torch_ev)
        elif DeviceEvent._hip.hipStreamWaitEvent(self._C.c_void_p(stream.cuda_stream), self._ev,
                                                 self._C.c_uint(0)) != 0:
            raise RuntimeError("hipStreamWaitEvent failed")


def copy_ceiling(torch, B, n_bytes, dev):
    """Plain streaming copy of n_bytes with the library's own copy kernel (GB/s read + written)."""
    n_copy = max(16, (n_bytes // 16) * 16)
    src = torch.empty(n_copy, dtype=torch.uint8, device=dev)
    dsts = [torch.empty(n_copy, dtype=torch.uint8, device=dev) for _ in range(2)]
    evc = new_events(torch, 20)
    for i in range(25):
        if i >= 5:
            evc[i - 5][0].record()
        B.mw_copy_bytes(dsts[i % 2], src, n_copy)
        if i >= 5:
            evc[i - 5][1].record()
    torch.cuda.synchronize()
    copy_ms = sum(a.elapsed_time(b) for a, b in evc) / len(evc)
    return {"GBps": round(2 * n_copy / copy_ms / 1e6, 1), "bytes": 2 * n_copy}


def traffic_from_profile(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE runs of this same command, scaled by what the plain copy kernel reads)."""
    path = os.path.join(ROOT, "profiles", "bench_%s_hbm_traffic.md" % workload)
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch %s:" % kernel):
                return int(line.split(":")[1])
    return None


# ------------------------------------------------------------------------------------------ dispatch
def bench_dispatch(args, name: str, brief: bool = False) -> dict:
    """brief: the step, its launch brackets and the per-kernel breakdown only (the per-configuration
    blocks of the default run); otherwise also the other schedules and the variants."""
    import numpy as np
    import torch
    from paper_2605_22428_amd import binding as B
    from paper_2605_22428_amd import workloads as W

    dev = "cuda:0"
    seed = W.BASE_SEED if args.seed is None else args.seed
    w = {"c0": W.C0, "c1": W.C1, "c2": W.C2, "c3": W.C3, "c3_hot": W.scaled(W.C3, n_tokens=512)}[name]
    my_rank = {"c3": W.zipf_median_rank(w, seed), "c3_hot": W.zipf_hottest_rank(w, seed)}.get(name, 0)
    pooled = name == "c3_hot"      # 114 k received rows: payload rows come from a pool (see workloads.payload_rows_pooled)
    sched0 = args.schedule
    if sched0 == "auto":
        # the plan of the next batch rides in the step's one launch where it stays in the row
        # movers' shadow (up to 4096 tokens); beyond that it runs on a second stream
        sched0 = "one_launch" if w.n_tokens <= 4096 else "launch_and_plan"
    describe = {
        "c0": "C0 tiny dispatch: 8 simulated ranks, 16 experts, top-2 uniform, 128 tokens x 256 bf16, 8 peer "
              "receive regions (launch-latency bound, cache resident: its % of peak is not meaningful)",
        "c1": "C1 DeepSeek-V3-shaped dispatch: 64 simulated ranks, 256 experts, top-8 group-limited (<=4 of 8 "
              "nodes), 4096 tokens x 7168 bf16 on this rank, 64 peer receive regions",
        "c2": "C2 = C1 with fp8 e4m3 payload + one fp32 scale per 128 elements (7392-byte rows)",
        "c3": "C3 large-EP skewed dispatch: 256 simulated ranks, 256 experts (1 per rank), 8192 tokens x 7168 "
              "bf16, top-8 Zipf(1.1); receive side at the rank of the median-popularity expert",
        "c3_hot": "C3 skew stress point: the rank of the most popular expert, 256 peers x 512 tokens x 7168 bf16, "
                  "top-8 Zipf(1.1) (this rank's own batch is 512 tokens too; payload rows drawn from a pool)",
    }[name]
    R, K, T, rb = w.n_ranks, w.top_k, w.n_tokens, w.row_bytes
    # rows that are not whole cache lines lie a whole number of lines apart in the packed and the
    # received arrays (mw_config.row_stride_bytes; fp8: 7392-byte rows every 7424 bytes): layout
    # only -- the bytes moved and counted are the rows' own
    stride = (rb + 127) // 128 * 128 if args.row_stride is None else args.row_stride
    e2r = W.expert_to_rank(w)
    L = w.experts_per_rank
    fp8 = w.row_format == "fp8"
    fmt = B.MW_ROW_FP8_E4M3_BLOCK128 if fp8 else B.MW_ROW_BF16
    xdt = torch.uint8 if fp8 else torch.int16

    def up(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(a).to(dev)

    # ---------------------------------------------------------------- set-up (untimed)
    t_setup = time.time()
    ctx = B.Context(R, w.n_experts, K, my_rank, w.hidden, fmt, T, R * T, e2r, device=dev, max_hops=16, row_stride=stride)
    ctx_b = B.Context(R, w.n_experts, K, my_rank, w.hidden, fmt, T, R * T, e2r, device=dev, row_stride=stride)   # second receive index
    ctx_p = B.Context(R, w.n_experts, K, my_rank, w.hidden, fmt, T, 1, e2r, device=dev, row_stride=stride)       # plans beside mw_stream_step
    topks = W.topk_ids_many(w, seed, range(R))
    def draw(p, tokens=None):
        return (W.payload_rows_pooled(w, seed, p, tokens), None) if pooled else W.payload_rows(w, seed, p, tokens)

    x_me, s_me = draw(my_rank)
    topk_d = up(topks[my_rank])
    log("[bench] routing and local payload drawn in %.1fs" % (time.time() - t_setup))

    # peer receive regions: every simulated peer's plan + pack + delivery runs on the GPU too
    x_peer = torch.zeros((T, w.hidden), dtype=xdt, device=dev)
    s_peer = torch.zeros((T, w.hidden // 128), dtype=torch.float32, device=dev) if fp8 else None
    sb = B.SendBuffers(ctx, T)
    out = dict(desc=torch.zeros((T, B.DESC_BYTES), dtype=torch.uint8, device=dev),
               rows=torch.zeros((T, stride), dtype=torch.uint8, device=dev),
               row_src_token=torch.zeros(T, dtype=torch.int32, device=dev),
               row_topk=torch.zeros((T, K), dtype=torch.int32, device=dev))
    counts = torch.zeros(2, dtype=torch.int32, device=dev)
    recs = []
    # the same peers' traffic as packets (header in front of every row), for the packet path
    with_packets = name in ("c1", "c2") and not brief
    hb = B.mw_packet_header_bytes(K)
    pk_all = torch.zeros((T, hb + rb), dtype=torch.uint8, device=dev) if with_packets else None
    pk_regions = []
    for p in range(R):
        tokens = W.tokens_for_rank(w, topks[p], my_rank)     # (which rows are worth drawing; checked below)
        rows, sc = draw(p, tokens)
        idx = torch.from_numpy(tokens).to(dev)
        x_peer.zero_()
        x_peer[idx] = up(rows).view(xdt)
        if fp8:
            s_peer.zero_()
            s_peer[idx] = up(sc)
        tk_d = up(topks[p])
        ctx.mw_plan(tk_d, sb.mask, sb.perm, sb.desc, sb.stats)
        ctx.mw_pack(x_peer, s_peer, tk_d, sb.perm, sb.stats, sb.packed, sb.row_src_token, sb.row_topk)
        ctx.mw_sim_deliver(sb.desc, sb.stats, T, sb.packed, sb.row_src_token, sb.row_topk, my_rank,
                           out["desc"], out["rows"], out["row_src_token"], out["row_topk"], counts)
        g, n = (int(v) for v in counts.cpu().numpy())
        assert n == len(tokens), "payload was drawn for other rows than those delivered"
        if with_packets:
            ctx.mw_pack_packets(x_peer, s_peer, tk_d, sb.mask, sb.perm, sb.stats, pk_all)
            n_p = int(ctx.mw_get_send_stats(sb.stats)["n_rows"])
            word = pk_all[:n_p, 8 * (my_rank >> 6): 8 * (my_rank >> 6) + 8].contiguous().view(torch.int64)[:, 0]
            pk_regions.append(pk_all[:n_p][((word >> (my_rank & 63)) & 1).bool()].clone())
        recs.append(dict(desc=out["desc"][:max(g, 1)].clone(), rows=out["rows"][:max(n, 1)].clone(),
                         row_src_token=out["row_src_token"][:max(n, 1)].clone(),
                         row_topk=out["row_topk"][:max(n, 1)].clone(), n_desc=g, n_rows=n))
    del x_peer, s_peer, out, pk_all
    M = sum(r["n_rows"] for r in recs)
    n_desc_total = sum(r["n_desc"] for r in recs)
    cap = max(1, M * min(K, L))

    sets = []
    for s in range(N_SETS):
        rs = [dict(desc=r["desc"].clone(), rows=r["rows"].clone(), row_src_token=r["row_src_token"].clone(),
                   row_topk=r["row_topk"].clone(), n_desc=r["n_desc"], n_rows=r["n_rows"]) for r in recs]
        sets.append(dict(x=up(x_me).view(xdt), sc=up(s_me) if fp8 else None, send=B.SendBuffers(ctx, T), recs=rs,
                         table=B.peers_table(rs, dev), recv=B.RecvBuffers(ctx, cap)))
    del recs
    torch.cuda.synchronize()
    log("[bench] %d peer regions built on the GPU, M=%d rows; set-up %.1fs" % (R, M, time.time() - t_setup))

    # The send side (plan, pack of this rank's tokens) and the receive side (unpack of what the
    # peers sent) are independent operations on disjoint buffers and disjoint workspace.
    s_send, s_recv = torch.cuda.Stream(), torch.cuda.Stream()
    for st_ in (s_send, s_recv):                 # both streams get their hardware queue now, not in the
        with torch.cuda.stream(st_):             # middle of the schedule comparison
            torch.zeros(1, device=dev)
    torch.cuda.synchronize()

    def send_side(s):
        sd = s["send"]
        ctx.mw_plan(topk_d, sd.mask, sd.perm, sd.desc, sd.stats)
        ctx.mw_pack(s["x"], s["sc"], topk_d, sd.perm, sd.stats, sd.packed, sd.row_src_token, sd.row_topk)

    def recv_side(s):
        rv = s["recv"]
        ctx.mw_unpack(s["table"], R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer, rv.out_src_token,
                      rv.expert_offsets, rv.stats)

    # Schedules of a step (all move the same bytes through the same kernels):
    #  "aligned"  the send side and the receive side are independent operations, each
    #            issued on its own stream; one cross-stream wait per step holds the packer back
    #            until the previous batch's expander has finished.  The packer (bandwidth-bound,
    #            short) then runs beside the receive index (latency-bound, moves almost nothing),
    #            the plan of the next batch (latency-bound) beside the expander, and the two
    #            bandwidth-bound kernels never share HBM: the expander's launches show its own rate.
    #  "free"    no wait: the two streams drift; when packer and expander overlap, an expander
    #            launch takes longer by about the packer's bytes.
    #  "single"  everything on one stream.
    #  "pipelined"  as "aligned", but the receive side is one launch per step
    #            (mw_unpack_expand_index_next): the expander of this batch with the index of the
    #            next batch riding along, on two contexts used alternately.  The latency-bound index
    #            no longer stands in front of its expander.  Every step still does one plan, one
    #            pack, one index and one expand; the first batch's index is built before the timed
    #            region (in steady state the step before builds it), the last step builds one that
    #            is not used.  The index is then hidden behind the expander, but the packer no longer
    #            has the index to hide behind: the step takes as long as in "aligned".
    #  "one_stream"  two launches per batch on ONE stream and no event: the packer, then
    #            mw_unpack_expand_index_plan_next -- the expander of this batch with the index AND the
    #            plan of the next batch riding along.  Nothing latency-bound stands alone any more,
    #            and nothing waits across streams.  Every step still does one plan, one pack, one
    #            index and one expand; the first batch's plan and index are made before the timed
    #            region, the last step makes ones that are not used.
    #  "launch_and_plan"  for batches whose plan would outlast the expander: mw_stream_step with an
    #            empty next batch to plan (packer, expander and the next index in one launch) and
    #            mw_plan of the real next batch on the second stream; the launch waits for the plan
    #            made during the step before, and the plan waits until the step that last packed
    #            from its output buffers (the same buffer set, N_SETS - 1 steps ago) has finished.
    #  "one_launch" (what "auto", the default, takes for batches of up to 4096 tokens; larger
    #            ones get "launch_and_plan")  mw_stream_step: the packer joins that launch too -- one
    #            launch per batch, the two bandwidth-bound parts with no launch boundary between
    #            them.  The launch's algorithmic bytes are then the packer's plus the expander's.
    ev_unpack_done = [DeviceEvent(torch) for _ in range(2)]
    ev_plan_done = [DeviceEvent(torch) for _ in range(2)]
    ev_step_done = [DeviceEvent(torch) for _ in range(N_SETS)]
    no_plan_stats = torch.zeros(B.SEND_STATS_BYTES, dtype=torch.uint8, device=dev)
    state = {"n": 0}
    rctx = [ctx, ctx_b]
    pipe = {"n": 0}
    step_records = {}
    s_recv_handle = s_recv.cuda_stream
    lap = {"n": 0}            # launch_and_plan steps issued since the pipeline was primed

    def prime_pipeline(with_plan=False):
        """Index (and, for "one_stream", plan) of the batch the next pipelined step works on; the
        other schedules use the same workspace in between."""
        n = pipe["n"]
        lap["n"] = 0
        s = sets[n % N_SETS]
        with torch.cuda.stream(s_recv):
            rctx[n % 2].mw_unpack_index(s["table"], R, cap, s["recv"].expert_offsets, s["recv"].stats)
            if with_plan:
                sd = s["send"]
                ctx.mw_plan(topk_d, sd.mask, sd.perm, sd.desc, sd.stats)
                ev_plan_done[n % 2].record(s_recv)

    def step(i: int, schedule: str = sched0):
        s = sets[i % N_SETS]
        if schedule == "single":
            send_side(s)
            recv_side(s)
        elif schedule == "free":
            with torch.cuda.stream(s_send):
                send_side(s)
            with torch.cuda.stream(s_recv):
                recv_side(s)
        elif schedule == "pipelined":
            n = pipe["n"]
            pipe["n"] = n + 1
            s, s_next = sets[n % N_SETS], sets[(n + 1) % N_SETS]
            sd, rv, rn = s["send"], s["recv"], s_next["recv"]
            with torch.cuda.stream(s_send):
                ctx.mw_plan(topk_d, sd.mask, sd.perm, sd.desc, sd.stats)
                if n > 0:
                    ev_unpack_done[(n - 1) % 2].make_wait(s_send)
                ctx.mw_pack(s["x"], s["sc"], topk_d, sd.perm, sd.stats, sd.packed, sd.row_src_token, sd.row_topk)
            with torch.cuda.stream(s_recv):
                rctx[n % 2].mw_unpack_expand_index_next(R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer,
                                                        rv.out_src_token, rctx[(n + 1) % 2], s_next["table"], R, cap,
                                                        rn.expert_offsets, rn.stats)
                ev_unpack_done[n % 2].record(s_recv)
        elif schedule == "one_stream":
            n = pipe["n"]
            pipe["n"] = n + 1
            s, s_next = sets[n % N_SETS], sets[(n + 1) % N_SETS]
            sd, rv, rn, sdn = s["send"], s["recv"], s_next["recv"], s_next["send"]
            with torch.cuda.stream(s_recv):
                ctx.mw_pack(s["x"], s["sc"], topk_d, sd.perm, sd.stats, sd.packed, sd.row_src_token, sd.row_topk)
                rctx[n % 2].mw_unpack_expand_index_plan_next(R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer,
                                                             rv.out_src_token, rctx[(n + 1) % 2], s_next["table"], R,
                                                             cap, rn.expert_offsets, rn.stats, topk_d, sdn.mask,
                                                             sdn.perm, sdn.desc, sdn.stats)
        elif schedule == "one_launch":
            n = pipe["n"]
            pipe["n"] = n + 1
            key = (n % N_SETS, n % 2)
            if key not in step_records:     # the batch records of this (buffer set, context) pair: built once
                s, s_next = sets[n % N_SETS], sets[(n + 1) % N_SETS]
                sd, rv, rn, sdn = s["send"], s["recv"], s_next["recv"], s_next["send"]
                step_records[key] = (B.send_batch(s["x"], s["sc"], topk_d, sd.perm, sd.stats, sd.packed, sd.row_src_token,
                                                  sd.row_topk),
                                     B.recv_batch(R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer, rv.out_src_token),
                                     B.next_batch(rctx[(n + 1) % 2], s_next["table"], R, cap, rn.expert_offsets, rn.stats,
                                                  topk_d, sdn.mask, sdn.perm, sdn.desc, sdn.stats))
            rctx[n % 2].mw_stream_step_records(*step_records[key], stream_handle=s_recv_handle)
        elif schedule == "launch_and_plan":
            n = pipe["n"]
            pipe["n"] = n + 1
            s, s_next = sets[n % N_SETS], sets[(n + 1) % N_SETS]
            sd, rv, rn, sdn = s["send"], s["recv"], s_next["recv"], s_next["send"]
            with torch.cuda.stream(s_send):                      # the plan of the next batch, beside the launch
                if lap["n"] >= N_SETS - 1:                       # its buffers: last packed from N_SETS - 1 steps ago
                    ev_step_done[(n + 1) % N_SETS].make_wait(s_send)
                ctx_p.mw_plan(topk_d, sdn.mask, sdn.perm, sdn.desc, sdn.stats)     # (its own context: the launch's
                                                                                   # empty plan uses ctx's or ctx_b's)
                ev_plan_done[(n + 1) % 2].record(s_send)
            with torch.cuda.stream(s_recv):
                ev_plan_done[n % 2].make_wait(s_recv)            # (made during the step before: long complete)
                rctx[n % 2].mw_stream_step(s["x"], s["sc"], topk_d, sd.perm, sd.stats, sd.packed, sd.row_src_token,
                                           sd.row_topk, R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer,
                                           rv.out_src_token, rctx[(n + 1) % 2], s_next["table"], R, cap,
                                           rn.expert_offsets, rn.stats, topk_d[:0], None, None, None, no_plan_stats)
                ev_step_done[n % N_SETS].record(s_recv)
            lap["n"] += 1
        else:
            n = state["n"]
            state["n"] = n + 1
            sd = s["send"]
            with torch.cuda.stream(s_send):
                ctx.mw_plan(topk_d, sd.mask, sd.perm, sd.desc, sd.stats)
                if n > 0:
                    ev_unpack_done[(n - 1) % 2].make_wait(s_send)
                ctx.mw_pack(s["x"], s["sc"], topk_d, sd.perm, sd.stats, sd.packed, sd.row_src_token, sd.row_topk)
            with torch.cuda.stream(s_recv):
                recv_side(s)
                ev_unpack_done[n % 2].record(s_recv)

    def set_expand_events(a, b):
        for c in rctx:
            c.mw_ctx_set_timing_events(B.MW_KERNEL_EXPAND, a, b)

    # ---------------------------------------------------------------- warm-up, then the timed region
    if sched0 in ("pipelined", "one_stream", "one_launch", "launch_and_plan"):
        prime_pipeline(sched0 != "pipelined")
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    st = ctx.mw_get_send_stats(sets[0]["send"].stats)
    rs0 = ctx.mw_get_recv_stats(sets[0]["recv"].stats)
    ctx_b.mw_get_recv_stats(sets[0]["recv"].stats)      # (both contexts size their launches from the rows seen)
    N, Q = int(st["n_rows"]), int(rs0["n_out_rows"])
    assert int(st["error_flags"]) == 0 and int(rs0["error_flags"]) == 0 and int(rs0["n_recv_rows"]) == M

    # An event pair costs a few microseconds of bubble on this platform, so the expander is
    # bracketed on every EV_STRIDE-th step of the timed region only.
    EV_STRIDE = 8
    ev_expand = new_events(torch, (args.steps + EV_STRIDE - 1) // EV_STRIDE)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % EV_STRIDE == 0:
            set_expand_events(*ev_expand[i // EV_STRIDE])
        elif i % EV_STRIDE == 1:
            set_expand_events(None, None)
        step(i)
    t_issued = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    set_expand_events(None, None)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    issue_ms_per_step = (t_issued - t0) * 1e3 / args.steps      # host time to enqueue a step
    region_ms = sorted(a.elapsed_time(b) for a, b in ev_expand)
    # A further pass of the same steps with EVERY launch bracketed (not part of the timed region:
    # the brackets' bubbles would be in `value`): the figures of the roofline block.
    n_br = max(24, min(args.steps, 64))
    ev_br = new_events(torch, n_br)
    for i in range(n_br):
        set_expand_events(*ev_br[i])
        step(args.steps + i)
    torch.cuda.synchronize()
    set_expand_events(None, None)
    expand_ms = sorted(a.elapsed_time(b) for a, b in ev_br)
    expand_avg_ms = sum(expand_ms) / len(expand_ms)
    expand_med_ms = 0.5 * (expand_ms[(len(expand_ms) - 1) // 2] + expand_ms[len(expand_ms) // 2])

    other, other_issue = {}, {}
    for sched in ("single", "free", "aligned", "pipelined", "one_stream", "one_launch", "launch_and_plan"):
        if sched == sched0 or brief:                        # the other schedules, for reference
            continue
        if sched in ("pipelined", "one_stream", "one_launch", "launch_and_plan"):
            prime_pipeline(sched != "pipelined")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i, sched)
        other_issue[sched] = round((time.perf_counter() - t0) * 1e3 / args.steps, 4)
        torch.cuda.synchronize()
        other[sched] = round((time.perf_counter() - t0) * 1e3 / args.steps, 4)

    # ---------------------------------------------------------------- per-kernel breakdown (one stream, untimed)
    names = {"plan_rank": B.MW_KERNEL_PLAN_RANK,
             "plan_groups": B.MW_KERNEL_PLAN_GROUPS, "pack": B.MW_KERNEL_PACK,
             "recv_index": B.MW_KERNEL_RECV_INDEX, "expand": B.MW_KERNEL_EXPAND}
    n_b = min(args.steps, 50)
    evs = {k: new_events(torch, n_b) for k in names}
    for i in range(n_b):
        for k, code in names.items():
            ctx.mw_ctx_set_timing_events(code, *evs[k][i])
        step(i, "single")
    torch.cuda.synchronize()
    for code in names.values():
        ctx.mw_ctx_set_timing_events(code, None, None)
    kern_us = {k: 1e3 * sum(a.elapsed_time(b) for a, b in evs[k]) / n_b for k in names}

    ceiling = copy_ceiling(torch, B, M * rb, dev)    # plain copy of as many bytes as one expand launch reads

    # ---------------------------------------------------------------- relay step (extra, untimed region)
    # This rank as the first relay of its own packed buffer in a two-level topology: servers
    # of 8 devices, direct links inside the server, one link per remote server (to its
    # same-index device).  One read of every row, one write per distinct next hop.
    relay = None
    if name in ("c1", "c2") and not brief:
        n_per = 8
        next_hop = np.array([(r % n_per) if r // n_per == my_rank // n_per else n_per + (r // n_per) -
                             (1 if r // n_per > my_rank // n_per else 0) for r in range(R)], dtype=np.int32)
        n_hops = n_per + R // n_per - 1
        ctx.mw_set_forwarding(next_hop, n_hops)
        children = B.RelayChildren(ctx, n_hops, T)
        sd0 = sets[0]["send"]
        in_rec = B.peers_table([dict(desc=sd0.desc, rows=sd0.packed, row_src_token=sd0.row_src_token,
                                     row_topk=sd0.row_topk, n_desc=int(st["n_groups"]), n_rows=N)], dev)
        relay_names = {"relay_index": B.MW_KERNEL_RELAY_INDEX, "relay_copy": B.MW_KERNEL_RELAY_COPY}
        n_r = 20
        evr = {k: new_events(torch, n_r) for k in relay_names}
        for i in range(n_r + 3):
            if i >= 3:
                for k, code in relay_names.items():
                    ctx.mw_ctx_set_timing_events(code, *evr[k][i - 3])
            ctx.mw_relay(in_rec, children.table, T, children.stats)
        torch.cuda.synchronize()
        for code in relay_names.values():
            ctx.mw_ctx_set_timing_events(code, None, None)
        rst = ctx.mw_get_relay_stats(children.stats)
        assert int(rst["error_flags"]) == 0 and int(rst["n_rows_in"]) == N
        relay_us = {k: 1e3 * sum(a.elapsed_time(b) for a, b in evr[k]) / n_r for k in relay_names}
        rows_fwd = int(rst["forward_bytes"]) // rb
        relay_bytes = N * rb + rows_fwd * rb + N * (4 + 4 * K) + rows_fwd * (4 + 4 * K)
        relay = {"workload": "rank 0 relays its own packed buffer: %d servers x 8 devices, %d next hops"
                             % (R // n_per, n_hops),
                 "us": {k: round(v, 2) for k, v in relay_us.items()},
                 "copies_per_row": round(rows_fwd / N, 4),
                 "bytes_saved_vs_unicast": round(1.0 - int(rst["forward_bytes"]) / int(rst["unicast_bytes"]), 4),
                 "copy_bytes": relay_bytes, "copy_GBps": round(relay_bytes / relay_us["relay_copy"] / 1e3, 1),
                 "copy_pct_of_hbm_peak": round(100.0 * relay_bytes / relay_us["relay_copy"] / 1e3 / HBM_PEAK_GBPS, 2)}
        # a stream of buffers: the index of the next buffer rides in the launch that copies this one
        # (two contexts in turn, their own children), against mw_relay call by call
        ctx_r = B.Context(R, w.n_experts, K, my_rank, w.hidden, fmt, T, 1, e2r, device=dev, max_hops=16, row_stride=stride)
        ctx_r.mw_set_forwarding(next_hop, n_hops)
        kids = [children, B.RelayChildren(ctx_r, n_hops, T)]
        rc = [ctx, ctx_r]
        n_s = 40
        for form in ("stream", "calls"):
            if form == "stream":
                ctx.mw_relay_index(in_rec, kids[0].table, T, kids[0].stats)
            for i in range(n_s + 4):
                if i == 4:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                if form == "stream":
                    rc[i % 2].mw_relay_copy_index_next(in_rec, kids[i % 2].table, kids[i % 2].stats, rc[(i + 1) % 2], in_rec,
                                                       kids[(i + 1) % 2].table, T, kids[(i + 1) % 2].stats)
                else:
                    rc[i % 2].mw_relay(in_rec, kids[i % 2].table, T, kids[i % 2].stats)
            torch.cuda.synchronize()
            relay["step_us_" + form] = round((time.perf_counter() - t0) * 1e6 / n_s, 2)
            if form == "stream":             # the buffer indexed by the last launch is copied too
                rc[(n_s + 4) % 2].mw_relay_copy(in_rec, kids[(n_s + 4) % 2].table, kids[(n_s + 4) % 2].stats)
        for c_, k_ in zip(rc, kids):
            rs_ = c_.mw_get_relay_stats(k_.stats)
            assert int(rs_["error_flags"]) == 0 and int(rs_["n_rows_in"]) == N and int(rs_["forward_bytes"]) == int(rst["forward_bytes"])
        relay["step_GBps_stream"] = round(relay_bytes / relay["step_us_stream"] / 1e3, 1)
        relay["step_pct_of_hbm_peak_stream"] = round(100.0 * relay_bytes / relay["step_us_stream"] / 1e3 / HBM_PEAK_GBPS, 2)
        # several buffers a launch (mw_relay_batch): NB copies and the next NB indexes, 2 NB contexts in turn
        for NB in (2, 4):
            cs = [ctx, ctx_r] + [B.Context(R, w.n_experts, K, my_rank, w.hidden, fmt, T, 1, e2r, device=dev, max_hops=16,
                                           row_stride=stride) for _ in range(2 * NB - 2)]
            for c_ in cs[2:]:
                c_.mw_set_forwarding(next_hop, n_hops)
            kb = kids + [B.RelayChildren(c_, n_hops, T) for c_ in cs[2:]]
            jobs = [B.relay_job(c_, in_rec, k_.table, T, k_.stats) for c_, k_ in zip(cs, kb)]
            for c_, k_ in zip(cs[:NB], kb[:NB]):
                c_.mw_relay_index(in_rec, k_.table, T, k_.stats)
            for i in range(n_s + 4):
                if i == 4:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                B.mw_relay_batch(*((jobs[:NB], jobs[NB:]) if i % 2 == 0 else (jobs[NB:], jobs[:NB])))
            torch.cuda.synchronize()
            per = (time.perf_counter() - t0) * 1e6 / n_s / NB
            B.mw_relay_batch(jobs[:NB] if (n_s + 4) % 2 == 0 else jobs[NB:], [])
            for c_, k_ in zip(cs, kb):
                rs_ = c_.mw_get_relay_stats(k_.stats)
                assert int(rs_["error_flags"]) == 0 and int(rs_["forward_bytes"]) == int(rst["forward_bytes"])
            relay["us_per_buffer_batch_of_%d" % NB] = round(per, 2)
            relay["pct_of_hbm_peak_batch_of_%d" % NB] = round(100.0 * relay_bytes / per / 1e3 / HBM_PEAK_GBPS, 2)
            for c_ in cs[2:]:
                c_.close()
            del kb, jobs
        ctx_r.close()
        del children, kids

    # ---------------------------------------------------------------- packet path (extra, untimed region)
    # The same step with the bitmap and the row metadata in a header in front of every row
    # (Section 6.4) instead of descriptor tables and side arrays.
    packets = None
    if with_packets:
        assert sum(int(r.shape[0]) for r in pk_regions) == M
        pk_table = B.packets_table(pk_regions, [int(r.shape[0]) for r in pk_regions], dev)
        pk_send = torch.zeros((T, hb + rb), dtype=torch.uint8, device=dev)
        s0 = sets[0]
        sd, rv = s0["send"], s0["recv"]
        pk_names = {"pack": B.MW_KERNEL_PACK, "recv_index": B.MW_KERNEL_RECV_INDEX, "expand": B.MW_KERNEL_EXPAND}
        n_r = 20
        evp = {k: new_events(torch, n_r) for k in pk_names}
        for i in range(n_r + 3):
            if i >= 3:
                for k, code in pk_names.items():
                    ctx.mw_ctx_set_timing_events(code, *evp[k][i - 3])
            ctx.mw_pack_packets(s0["x"], s0["sc"], topk_d, sd.mask, sd.perm, sd.stats, pk_send)
            ctx.mw_unpack_packets(pk_table, R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer, rv.out_src_token,
                                  rv.expert_offsets, rv.stats)
        torch.cuda.synchronize()
        for code in pk_names.values():
            ctx.mw_ctx_set_timing_events(code, None, None)
        rsp = ctx.mw_get_recv_stats(rv.stats)
        assert int(rsp["error_flags"]) == 0 and int(rsp["n_recv_rows"]) == M and int(rsp["n_out_rows"]) == Q
        pk_us = {k: 1e3 * sum(a.elapsed_time(b) for a, b in evp[k]) / n_r for k in pk_names}
        pk_pack_bytes = N * rb + N * (hb + rb) + N * (4 * K + 32 + 4)
        pk_expand_bytes = M * rb + Q * rb + Q * 8 + M * 4
        packets = {"header_bytes": hb, "overhead_pct_of_row": round(100.0 * hb / rb, 3),
                   "us": {k: round(v, 2) for k, v in pk_us.items()},
                   "pack_GBps": round(pk_pack_bytes / pk_us["pack"] / 1e3, 1),
                   "expand_GBps": round(pk_expand_bytes / pk_us["expand"] / 1e3, 1),
                   "expand_pct_of_hbm_peak": round(100.0 * pk_expand_bytes / pk_us["expand"] / 1e3 / HBM_PEAK_GBPS, 2)}
        # the relay step on this rank's own packets, same two-level topology as above
        kids = [torch.zeros((T, hb + rb), dtype=torch.uint8, device=dev) for _ in range(n_hops)]
        kid_table = torch.tensor([k.data_ptr() for k in kids], dtype=torch.int64, device=dev)
        in_pk = B.packets_table([pk_send], [N], dev)
        rstats = torch.zeros(B.RELAY_STATS_BYTES, dtype=torch.uint8, device=dev)
        evr = {k: new_events(torch, n_r) for k in relay_names}
        for i in range(n_r + 3):
            if i >= 3:
                for k, code in relay_names.items():
                    ctx.mw_ctx_set_timing_events(code, *evr[k][i - 3])
            ctx.mw_relay_packets(in_pk, kid_table, T, rstats)
        torch.cuda.synchronize()
        for code in relay_names.values():
            ctx.mw_ctx_set_timing_events(code, None, None)
        rst = ctx.mw_get_relay_stats(rstats)
        assert int(rst["error_flags"]) == 0 and int(rst["n_rows_in"]) == N
        rp_us = {k: 1e3 * sum(a.elapsed_time(b) for a, b in evr[k]) / n_r for k in relay_names}
        rp_bytes = N * (hb + rb) + int(rst["forward_bytes"])
        packets["relay"] = {"us": {k: round(v, 2) for k, v in rp_us.items()},
                            "copies_per_packet": round(int(rst["forward_bytes"]) / (hb + rb) / N, 4),
                            "copy_GBps": round(rp_bytes / rp_us["relay_copy"] / 1e3, 1)}
        # a stream of packet buffers on two contexts against mw_relay_packets call by call
        ctx_r = B.Context(R, w.n_experts, K, my_rank, w.hidden, fmt, T, 1, e2r, device=dev, max_hops=16, row_stride=stride)
        ctx_r.mw_set_forwarding(next_hop, n_hops)
        kids2 = [torch.zeros((T, hb + rb), dtype=torch.uint8, device=dev) for _ in range(n_hops)]
        tabs = [kid_table, torch.tensor([k.data_ptr() for k in kids2], dtype=torch.int64, device=dev)]
        sts, rc = [rstats, torch.zeros_like(rstats)], [ctx, ctx_r]
        n_s = 40
        for form in ("stream", "calls"):
            if form == "stream":
                ctx.mw_relay_packets_index(in_pk, T, sts[0])
            for i in range(n_s + 4):
                if i == 4:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                if form == "stream":
                    rc[i % 2].mw_relay_packets_copy_index_next(in_pk, tabs[i % 2], sts[i % 2], rc[(i + 1) % 2], in_pk, T,
                                                               sts[(i + 1) % 2])
                else:
                    rc[i % 2].mw_relay_packets(in_pk, tabs[i % 2], T, sts[i % 2])
            torch.cuda.synchronize()
            packets["relay"]["step_us_" + form] = round((time.perf_counter() - t0) * 1e6 / n_s, 2)
            if form == "stream":             # the buffer indexed by the last launch is copied too
                rc[(n_s + 4) % 2].mw_relay_packets_copy(in_pk, tabs[(n_s + 4) % 2], sts[(n_s + 4) % 2])
        for c_, s_ in zip(rc, sts):
            rs_ = c_.mw_get_relay_stats(s_)
            assert int(rs_["error_flags"]) == 0 and int(rs_["forward_bytes"]) == int(rst["forward_bytes"])
        packets["relay"]["step_GBps_stream"] = round(rp_bytes / packets["relay"]["step_us_stream"] / 1e3, 1)
        ctx_r.close()
        del pk_send, pk_table, kids, kids2
    del pk_regions

    # ---------------------------------------------------------------- quantise-in-pack (extra, untimed region)
    # fp8 workload only: the packer fed with this rank's bf16 rows, quantising on the way.
    quant = None
    if fp8 and not brief:
        import dataclasses
        xb, _ = W.payload_rows(dataclasses.replace(w, row_format="bf16"), seed, my_rank)
        xb_d = up(xb)
        sd = sets[0]["send"]
        n_r = 20
        evq = new_events(torch, n_r)
        for i in range(n_r + 3):
            if i >= 3:
                ctx.mw_ctx_set_timing_events(B.MW_KERNEL_PACK_QUANT, *evq[i - 3])
            ctx.mw_pack_quantize(xb_d, topk_d, sd.perm, sd.stats, sd.packed, sd.row_src_token, sd.row_topk)
        torch.cuda.synchronize()
        ctx.mw_ctx_set_timing_events(B.MW_KERNEL_PACK_QUANT, None, None)
        q_us = 1e3 * sum(a.elapsed_time(b) for a, b in evq) / n_r
        q_bytes = N * 2 * w.hidden + N * rb + N * (4 + 4 * K) + N * 4 + N * 4 * K
        quant = {"us": round(q_us, 2), "bytes": q_bytes, "GBps": round(q_bytes / q_us / 1e3, 1),
                 "pct_of_hbm_peak": round(100.0 * q_bytes / q_us / 1e3 / HBM_PEAK_GBPS, 2),
                 "bytes_of_quantise_then_pack": q_bytes + 2 * N * rb}
        del xb_d

    # ---------------------------------------------------------------- the way back (extra, untimed region)
    # bf16 workloads: one returned row per received row, the sum of its local experts' outputs
    # (here: the expanded rows themselves stand in for the experts' outputs).
    combine = None
    if not fp8 and not brief:
        rv = sets[0]["recv"]
        ctx.mw_unpack(sets[0]["table"], R, rv.out_rows, rv.out_scales, cap, rv.out_src_peer, rv.out_src_token,
                      rv.expert_offsets, rv.stats)
        ret = torch.zeros((M, w.hidden), dtype=torch.int16, device=dev)
        n_r = 20
        evc = new_events(torch, n_r)
        for i in range(n_r + 3):
            if i >= 3:
                ctx.mw_ctx_set_timing_events(B.MW_KERNEL_COMBINE, *evc[i - 3])
            ctx.mw_combine_gather(R, rv.out_rows, cap, ret, M)
        torch.cuda.synchronize()
        ctx.mw_ctx_set_timing_events(B.MW_KERNEL_COMBINE, None, None)
        c_us = 1e3 * sum(a.elapsed_time(b) for a, b in evc) / n_r
        c_bytes = Q * rb + M * rb + M * 32
        combine = {"us": round(c_us, 2), "bytes": c_bytes, "GBps": round(c_bytes / c_us / 1e3, 1),
                   "pct_of_hbm_peak": round(100.0 * c_bytes / c_us / 1e3 / HBM_PEAK_GBPS, 2),
                   "rows_back": M, "rows_without_local_sum": Q}
        del ret

    # ---------------------------------------------------------------- decode-sized send side (extra, untimed region)
    # The first 64 / 128 tokens of this rank's batch (the small batch sizes of the paper's
    # dispatch experiment, Section 6.3): mw_plan + mw_pack against the single launch of
    # mw_plan_pack, back to back on one stream; and mw_unpack of what the peers send for batches
    # of that size.
    decode = {}
    sd0 = sets[0]["send"]
    for Td in (64, 128):
        if Td > T or brief:
            continue
        tk_s, x_s = topk_d[:Td], sets[0]["x"][:Td]
        sc_s = sets[0]["sc"][:Td] if fp8 else None

        def two_calls():
            ctx.mw_plan(tk_s, sd0.mask, sd0.perm, sd0.desc, sd0.stats)
            ctx.mw_pack(x_s, sc_s, tk_s, sd0.perm, sd0.stats, sd0.packed, sd0.row_src_token, sd0.row_topk)

        def one_launch():
            ctx.mw_plan_pack(tk_s, x_s, sc_s, sd0.mask, sd0.perm, sd0.desc, sd0.stats, sd0.packed,
                             sd0.row_src_token, sd0.row_topk)

        us = {}
        for label, fn in (("plan_then_pack_us", two_calls), ("plan_pack_us", one_launch)):
            for _ in range(10):
                fn()
            (a, b), = new_events(torch, 1)
            a.record()
            for _ in range(100):
                fn()
            b.record()
            torch.cuda.synchronize()
            us[label] = round(10.0 * a.elapsed_time(b), 2)
        # the receive side of the same batch size: every peer sends its first Td tokens
        ctx_d = B.Context(R, w.n_experts, K, my_rank, w.hidden, fmt, Td, R * Td, e2r, device=dev, row_stride=stride)
        sb_d = B.SendBuffers(ctx_d, Td)
        x_d = torch.zeros((Td, w.hidden), dtype=xdt, device=dev)
        s_d = torch.zeros((Td, w.hidden // 128), dtype=torch.float32, device=dev) if fp8 else None
        o_d = dict(desc=torch.zeros((Td, B.DESC_BYTES), dtype=torch.uint8, device=dev),
                   rows=torch.zeros((Td, stride), dtype=torch.uint8, device=dev),
                   row_src_token=torch.zeros(Td, dtype=torch.int32, device=dev),
                   row_topk=torch.zeros((Td, K), dtype=torch.int32, device=dev))
        recs_d = []
        for p in range(R):
            tk_p = up(topks[p][:Td])
            ctx_d.mw_plan_pack(tk_p, x_d, s_d, sb_d.mask, sb_d.perm, sb_d.desc, sb_d.stats, sb_d.packed,
                               sb_d.row_src_token, sb_d.row_topk)
            ctx_d.mw_sim_deliver(sb_d.desc, sb_d.stats, Td, sb_d.packed, sb_d.row_src_token, sb_d.row_topk, my_rank,
                                 o_d["desc"], o_d["rows"], o_d["row_src_token"], o_d["row_topk"], counts)
            g_d, n_d = (int(v) for v in counts.cpu().numpy())
            recs_d.append(dict(desc=o_d["desc"][:max(g_d, 1)].clone(), rows=o_d["rows"][:max(n_d, 1)].clone(),
                               row_src_token=o_d["row_src_token"][:max(n_d, 1)].clone(),
                               row_topk=o_d["row_topk"][:max(n_d, 1)].clone(), n_desc=g_d, n_rows=n_d))
        m_d = sum(r["n_rows"] for r in recs_d)
        cap_d = max(1, m_d * min(K, L))
        table_d, rv_d = B.peers_table(recs_d, dev), B.RecvBuffers(ctx_d, cap_d)

        def unpack_d():
            ctx_d.mw_unpack(table_d, R, rv_d.out_rows, rv_d.out_scales, cap_d, rv_d.out_src_peer, rv_d.out_src_token,
                            rv_d.expert_offsets, rv_d.stats)

        unpack_d()
        ctx_d.mw_get_recv_stats(rv_d.stats)
        for _ in range(10):
            unpack_d()
        (a, b), = new_events(torch, 1)
        a.record()
        for _ in range(100):
            unpack_d()
        b.record()
        torch.cuda.synchronize()
        us["unpack_us"] = round(10.0 * a.elapsed_time(b), 2)
        us["rows_received"] = m_d

        # a whole decode-sized step (send side, then receive side: three launches) issued call by
        # call, and the same three launches captured once into a HIP graph and replayed
        def step_d():
            one_launch()
            unpack_d()

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step_d()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step_d()
        # and as two launches: the packer, then the expander with the next batch's index and plan
        ctx_d2 = B.Context(R, w.n_experts, K, my_rank, w.hidden, fmt, Td, R * Td, e2r, device=dev, row_stride=stride)
        rv_d2 = B.RecvBuffers(ctx_d2, cap_d)
        ride_ctx, ride_rv, ride_n = (ctx_d, ctx_d2), (rv_d, rv_d2), {"n": 0}
        ctx_d2.mw_unpack_index(table_d, R, cap_d, rv_d2.expert_offsets, rv_d2.stats)
        ctx_d2.mw_get_recv_stats(rv_d2.stats)
        ctx_d.mw_unpack_index(table_d, R, cap_d, rv_d.expert_offsets, rv_d.stats)
        ctx_d.mw_plan(tk_s, sd0.mask, sd0.perm, sd0.desc, sd0.stats)

        def step_ride():
            n = ride_n["n"]
            ride_n["n"] = n + 1
            a, b = n % 2, (n + 1) % 2
            ctx.mw_pack(x_s, sc_s, tk_s, sd0.perm, sd0.stats, sd0.packed, sd0.row_src_token, sd0.row_topk)
            ride_ctx[a].mw_unpack_expand_index_plan_next(R, ride_rv[a].out_rows, ride_rv[a].out_scales, cap_d,
                                                         ride_rv[a].out_src_peer, ride_rv[a].out_src_token,
                                                         ride_ctx[b], table_d, R, cap_d, ride_rv[b].expert_offsets,
                                                         ride_rv[b].stats, tk_s, sd0.mask, sd0.perm, sd0.desc,
                                                         sd0.stats)

        # and as ONE launch (mw_stream_step); the plan riding in step n is the one step n + 1 packs from
        sd_pair = (sd0, B.SendBuffers(ctx, Td))
        for sd_ in sd_pair:
            ctx.mw_plan(tk_s, sd_.mask, sd_.perm, sd_.desc, sd_.stats)

        # (the batch records are built once: the loop marshals nothing, as a C caller's would not)
        recs_one = []
        for a in (0, 1):
            b = 1 - a
            recs_one.append((B.send_batch(x_s, sc_s, tk_s, sd_pair[a].perm, sd_pair[a].stats, sd_pair[a].packed,
                                          sd_pair[a].row_src_token, sd_pair[a].row_topk),
                             B.recv_batch(R, ride_rv[a].out_rows, ride_rv[a].out_scales, cap_d, ride_rv[a].out_src_peer,
                                          ride_rv[a].out_src_token),
                             B.next_batch(ride_ctx[b], table_d, R, cap_d, ride_rv[b].expert_offsets, ride_rv[b].stats,
                                          tk_s, sd_pair[b].mask, sd_pair[b].perm, sd_pair[b].desc, sd_pair[b].stats)))

        def step_one():
            n = ride_n["n"]
            ride_n["n"] = n + 1
            ride_ctx[n % 2].mw_stream_step_records(*recs_one[n % 2])

        for label, fn in (("step_us", step_d), ("step_graph_replay_us", graph.replay),
                          ("step_two_launches_us", step_ride), ("step_one_launch_us", step_one)):
            for _ in range(10):
                fn()
            (a, b), = new_events(torch, 1)
            a.record()
            for _ in range(100):
                fn()
            b.record()
            torch.cuda.synchronize()
            us[label] = round(10.0 * a.elapsed_time(b), 2)
        del graph
        ctx_d2.close()
        decode["%d_tokens" % Td] = us
        ctx_d.close()

    # ---------------------------------------------------------------- algorithmic bytes
    pack_bytes = 2 * N * rb + N * (4 + 4 * K) + N * 4 + N * 4 * K
    unpack_bytes = M * rb + Q * rb + M * (4 + 4 * K) + n_desc_total * 48 + Q * 8 + (L + 1) * 8
    expand_bytes = M * rb + Q * rb + Q * 8 + M * 4
    value = (pack_bytes + unpack_bytes) / (ms_per_step * 1e-3) / 1e9
    # the bracketed launch moves the expander's bytes -- and the packer's too in "one_launch"
    launch_bytes = expand_bytes + (pack_bytes if sched0 in ("one_launch", "launch_and_plan") else 0)
    achieved = launch_bytes / (expand_avg_ms * 1e-3) / 1e9
    pu_us = kern_us["pack"] + kern_us["recv_index"] + kern_us["expand"]
    saved = 1.0 - int(st["multicast_bytes"]) / int(st["unicast_bytes"])
    # the same figure without this rank's own copy (Section 3.1's AllGather counts the OTHER nodes
    # only): rows that go nowhere else are not sent at all, and no row counts its local copy
    G = int(st["n_groups"])
    desc_h = sets[0]["send"].desc.cpu().numpy().reshape(-1).view(B.DESC_DTYPE)[:G]
    own = np.zeros(4, dtype=np.uint64)
    own[my_rank >> 6] = np.uint64(1) << np.uint64(my_rank & 63)
    self_only_rows = int(desc_h["row_count"][(desc_h["mask"] == own).all(axis=1)].sum())
    copies = int(st["unicast_bytes"]) // rb
    to_others = copies - int(st["rows_per_dest"][my_rank])
    saved_excl_self = (1.0 - (N - self_only_rows) / to_others) if to_others > 0 else 0.0
    # cross-check straight from the routing table: per token, the distinct ranks other than this one
    tk_me = np.asarray(topks[my_rank])
    dest = np.where(tk_me >= 0, np.asarray(e2r)[np.clip(tk_me, 0, None)], -1)
    n_others = [len(set(int(r) for r in row if r >= 0 and r != my_rank)) for row in dest]
    assert to_others == sum(n_others) and N - self_only_rows == sum(1 for c in n_others if c > 0)

    # the launch that moves the receive side's bytes: the expander, in the pipelined schedule with
    # the next batch's index riding along (same bytes; the index's few MB are not counted)
    dominant = {"pipelined": "k_expand_index_next", "one_stream": "k_expand_index_plan_next",
                "one_launch": "k_expand_index_plan_next",
                "launch_and_plan": "k_expand_index_plan_next"}.get(sched0, "k_expand")
    payload = "fp8 e4m3 codes + fp32 scales, moved as bytes" if fp8 else "bf16 payload, moved as bytes"
    traffic_key = "mw_stream_step" if sched0 in ("one_launch", "launch_and_plan") else dominant
    traffic = traffic_from_profile(traffic_key, name.upper())
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": traffic,
                "traffic_source": None if traffic is None else
                "profiles/bench_%s_hbm_traffic.md: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                "not measured in this run" % name.upper(),
                "bytes_per_launch": launch_bytes,
                "avg_launch_ms": round(expand_avg_ms, 4), "median_launch_ms": round(expand_med_ms, 4),
                "min_launch_ms": round(expand_ms[0], 4), "launches_timed": len(expand_ms),
                "frac_of_median": round(launch_bytes / (expand_med_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "brackets": "every launch of a pass of %d steps that follows the timed region" % len(expand_ms),
                "in_timed_region": {"avg_launch_ms": round(sum(region_ms) / len(region_ms), 4),
                                    "launches_timed": len(region_ms)}}
    result = {
        "metric": METRIC,
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": payload, "data": "synthetic",
        "config": {"workload": describe, "seed": seed, "my_rank": my_rank,
                   "rows_packed": N, "groups": int(st["n_groups"]), "rows_received": M, "rows_out": Q,
                   "buffer_sets": N_SETS, "schedule": sched0, "row_bytes": rb, "row_stride_bytes": stride,
                   "streams": 1 if sched0 in ("single", "one_stream", "one_launch") else 2},
        "other_schedules_ms_per_step": other,
        "host_issue_ms_per_step": dict(other_issue, **{sched0: round(issue_ms_per_step, 4)}),
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "bytes_saved_vs_unicast": round(saved, 4),
        "bytes_saved_vs_unicast_excluding_self": round(saved_excl_self, 4),
        "step_bytes": {"pack": pack_bytes, "unpack": unpack_bytes},
        "kernel_us": {k: round(v, 2) for k, v in kern_us.items()},
        "pack_unpack_only": {"us": round(pu_us, 2),
                             "GBps": round((pack_bytes + unpack_bytes) / pu_us / 1e3, 1),
                             "pct_of_hbm_peak": round(100.0 * (pack_bytes + unpack_bytes) / pu_us / 1e3 / HBM_PEAK_GBPS, 2)},
        "copy_ceiling": ceiling,
        "roofline": roofline,
    }
    if brief:
        for c in (ctx, ctx_b, ctx_p):
            c.close()
        return {"workload": describe, "schedule": sched0, "dtype": payload, "steps": args.steps, "warmup": args.warmup,
                "rows": {"packed": N, "received": M, "out": Q},
                "ms_per_step": result["ms_per_step"], "GBps": result["value"],
                "pct_of_hbm_peak": result["pct_of_hbm_peak"],
                "bytes_saved_vs_unicast": result["bytes_saved_vs_unicast"],
                "step_bytes": result["step_bytes"], "kernel_us": result["kernel_us"],
                "pack_unpack_only": result["pack_unpack_only"], "copy_ceiling_GBps": ceiling["GBps"],
                "roofline": roofline}
    if relay is not None:
        result["relay"] = relay
    if decode:
        result["decode_sized_batches"] = decode
    if packets is not None:
        result["packets"] = packets
    if quant is not None:
        result["quantize_in_pack"] = quant
    if combine is not None:
        result["combine_gather"] = combine

    # ---------------------------------------------------------------- oracle on the host cores
    if not args.no_cpu_baseline and name == "c1":
        from oracle import ref
        log("[bench] cpu_baseline: building the oracle's own peer regions ...")
        bufs = []
        for p in range(R):
            tokens = W.tokens_for_rank(w, topks[p], my_rank)
            xp, _ = W.payload_full(w, seed, p, tokens)
            _, perm, desc, _ = ref.plan(topks[p], e2r, R, rb)
            packed, src_t, rtk = ref.pack(xp, None, topks[p], perm)
            bufs.append(ref.deliver(desc, packed, src_t, rtk, my_rank))
            del xp, packed
        reps, spent = 0, 0.0
        t_plan = t_pack = t_unpack = 0.0
        while reps < 3 or (spent < 12.0 and reps < 400):
            a = time.perf_counter()
            _, perm, desc, ost = ref.plan(topks[my_rank], e2r, R, rb)
            b = time.perf_counter()
            ref.pack(x_me, None, topks[my_rank], perm)
            c = time.perf_counter()
            o = ref.unpack(bufs, K, e2r, my_rank, rb, 0, cap)
            d = time.perf_counter()
            t_plan += b - a; t_pack += c - b; t_unpack += d - c
            spent += d - a; reps += 1
        assert len(o[2]) == Q and int(ost["n_rows"]) == N
        result["cpu_baseline"] = {
            "value": round((pack_bytes + unpack_bytes) * reps / (t_plan + t_pack + t_unpack) / 1e9, 3),
            "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "the whole C1 step (plan + pack of 4096 tokens, unpack of 64 peer regions), "
                      "%d repetitions, %.1f s of CPU time" % (reps, spent),
            "ms_per_step": round(1e3 * spent / reps, 2),
            "ms": {"plan": round(1e3 * t_plan / reps, 2), "pack": round(1e3 * t_pack / reps, 2),
                   "unpack": round(1e3 * t_unpack / reps, 2)},
            "host_cores_visible": os.cpu_count()}
        # the same step on all host cores: one independent step per thread (the oracle is single-threaded
        # as written and stays so; its C routines run outside the interpreter lock)
        from concurrent.futures import ThreadPoolExecutor
        n_thr = max(1, min(int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or 16, os.cpu_count() or 1, 16))
        step_s = spent / reps
        rounds = max(1, min(6, int(6.0 / max(step_s, 1e-3))))

        def one_step(_):
            _, perm_, _, _ = ref.plan(topks[my_rank], e2r, R, rb)
            ref.pack(x_me, None, topks[my_rank], perm_)
            return len(ref.unpack(bufs, K, e2r, my_rank, rb, 0, cap)[2])

        a = time.perf_counter()
        with ThreadPoolExecutor(n_thr) as ex:
            qs = list(ex.map(one_step, range(n_thr * rounds)))
        wall = time.perf_counter() - a
        assert all(q == Q for q in qs)
        result["cpu_baseline"]["all_cores"] = {
            "value": round((pack_bytes + unpack_bytes) * len(qs) / wall / 1e9, 3), "unit": "GB/s", "cores": n_thr,
            "sample": "%d independent C1 steps, one per thread at a time on %d threads, %.1f s wall"
                      % (len(qs), n_thr, wall)}

    for c in (ctx, ctx_b, ctx_p):
        c.close()
    return result


# ------------------------------------------------------------------------------------------ AllGather
def bench_allgather(args, brief: bool = False) -> dict:
    import numpy as np
    import torch
    from paper_2605_22428_amd import binding as B
    from paper_2605_22428_amd import workloads as W

    dev = "cuda:0"
    seed = W.BASE_SEED if args.seed is None else args.seed
    w = W.C4
    R, sbytes = w.n_ranks, w.shard_bytes
    ctx = B.Context(R, 0, 1, w.my_rank, 0, B.MW_ROW_BYTES, 1, R, None, row_bytes=sbytes, device=dev)
    shard = torch.from_numpy(W.allgather_shard(w, seed, w.my_rank).view(np.int16)).to(dev)
    # received shards: all ranks' (own included), three rotating sets
    sets = []
    for s in range(N_SETS):
        shards = [torch.from_numpy(W.allgather_shard(w, seed, r).view(np.int16)).to(dev) for r in range(R)]
        ptrs = torch.tensor([t.data_ptr() for t in shards], dtype=torch.int64, device=dev)
        sets.append(dict(shards=shards, ptrs=ptrs, send=torch.empty(sbytes, dtype=torch.uint8, device=dev),
                         desc=torch.zeros(B.DESC_BYTES, dtype=torch.uint8, device=dev),
                         stats=torch.zeros(B.SEND_STATS_BYTES, dtype=torch.uint8, device=dev),
                         out=torch.empty(R * sbytes, dtype=torch.uint8, device=dev)))
    torch.cuda.synchronize()

    # "one_launch" (auto): mw_allgather_step -- the shards received for one operation are
    # assembled while this rank's shard of the next one is loaded into its send buffer and
    # planned, in one launch; "single": the three calls one after the other.
    sched = "one_launch" if args.schedule in ("auto", "one_launch") else "single"

    def step_three(i):
        s = sets[i % N_SETS]
        ctx.mw_plan_allgather(sbytes, s["desc"], s["stats"])
        ctx.mw_pack_allgather(shard, sbytes, s["send"])
        ctx.mw_unpack_allgather(s["ptrs"], sbytes, s["out"])

    def step_one(i):
        s, sn = sets[i % N_SETS], sets[(i + 1) % N_SETS]
        ctx.mw_allgather_step(shard, sbytes, sn["send"], sn["desc"], sn["stats"], s["ptrs"], s["out"])

    step = step_one if sched == "one_launch" else step_three
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    st = ctx.mw_get_send_stats(sets[0]["stats"])
    EV_STRIDE = 4
    ev = new_events(torch, (args.steps + EV_STRIDE - 1) // EV_STRIDE)
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % EV_STRIDE == 0:
            ctx.mw_ctx_set_timing_events(B.MW_KERNEL_AG_GATHER, *ev[i // EV_STRIDE])
        elif i % EV_STRIDE == 1:
            ctx.mw_ctx_set_timing_events(B.MW_KERNEL_AG_GATHER, None, None)
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ctx.mw_ctx_set_timing_events(B.MW_KERNEL_AG_GATHER, None, None)
    region_ms = sorted(a.elapsed_time(b) for a, b in ev)
    # a further pass with every launch bracketed (outside the timed region): the roofline's figures
    n_br = max(24, min(args.steps, 64))
    ev_br = new_events(torch, n_br)
    for i in range(n_br):
        ctx.mw_ctx_set_timing_events(B.MW_KERNEL_AG_GATHER, *ev_br[i])
        step(args.steps + i)
    torch.cuda.synchronize()
    ctx.mw_ctx_set_timing_events(B.MW_KERNEL_AG_GATHER, None, None)
    g_ms = sorted(a.elapsed_time(b) for a, b in ev_br)
    g_avg = sum(g_ms) / len(g_ms)
    g_med = 0.5 * (g_ms[(len(g_ms) - 1) // 2] + g_ms[len(g_ms) // 2])
    names = {"pack_copy": B.MW_KERNEL_AG_PACK, "gather": B.MW_KERNEL_AG_GATHER}
    n_b = min(args.steps, 50)
    evs = {k: new_events(torch, n_b) for k in names}
    for i in range(n_b):
        for k, code in names.items():
            ctx.mw_ctx_set_timing_events(code, *evs[k][i])
        step_three(i)
    torch.cuda.synchronize()
    for code in names.values():
        ctx.mw_ctx_set_timing_events(code, None, None)
    kern_us = {k: 1e3 * sum(a.elapsed_time(b) for a, b in evs[k]) / n_b for k in names}
    pack_bytes, unpack_bytes = 2 * sbytes, 2 * R * sbytes
    value = (pack_bytes + unpack_bytes) / (ms_per_step * 1e-3) / 1e9
    launch_bytes = unpack_bytes + (pack_bytes if sched == "one_launch" else 0)
    achieved = launch_bytes / (g_avg * 1e-3) / 1e9
    other_step = step_three if sched == "one_launch" else step_one
    for i in range(5):
        other_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        other_step(i)
    torch.cuda.synchronize()
    other = {("single" if sched == "one_launch" else "one_launch"): round((time.perf_counter() - t0) * 1e3 / args.steps, 4)}
    traffic = traffic_from_profile("k_allgather_step" if sched == "one_launch" else "k_gather_shards", "C4")
    result = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 payload, moved as bytes", "data": "synthetic",
        "config": {"workload": "C4 AllGather receive assembly: 128-rank group, 2 MiB bf16 shard per rank, one "
                               "descriptor naming all ranks, 128 received shards -> 256 MiB in rank order "
                               "(the 4 MiB pack is launch-latency bound)", "seed": seed, "buffer_sets": N_SETS,
                   "schedule": sched, "streams": 1},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "bytes_saved_vs_unicast": round(1.0 - int(st["multicast_bytes"]) / int(st["unicast_bytes"]), 4),
        "step_bytes": {"pack": pack_bytes, "unpack": unpack_bytes},
        "ms_per_step_other_schedules": other,
        "kernel_us": {k: round(v, 2) for k, v in kern_us.items()},
        "copy_ceiling": copy_ceiling(torch, B, R * sbytes, dev),
        "roofline": {"kernel": "k_allgather_step" if sched == "one_launch" else "k_gather_shards",
                     "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic,
                     "traffic_source": None if traffic is None else
                     "profiles/bench_C4_hbm_traffic.md: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                     "command, not measured in this run",
                     "bytes_per_launch": launch_bytes,
                     "avg_launch_ms": round(g_avg, 4), "median_launch_ms": round(g_med, 4),
                     "min_launch_ms": round(g_ms[0], 4), "launches_timed": len(g_ms),
                     "frac_of_median": round(launch_bytes / (g_med * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                     "brackets": "every launch of a pass of %d steps that follows the timed region" % len(g_ms),
                     "in_timed_region": {"avg_launch_ms": round(sum(region_ms) / len(region_ms), 4),
                                         "launches_timed": len(region_ms)}},
    }
    if brief:
        result = {"workload": result["config"]["workload"], "schedule": sched, "dtype": result["dtype"],
                  "steps": args.steps, "warmup": args.warmup, "ms_per_step": result["ms_per_step"], "GBps": result["value"],
                  "pct_of_hbm_peak": result["pct_of_hbm_peak"],
                  "bytes_saved_vs_unicast": result["bytes_saved_vs_unicast"], "step_bytes": result["step_bytes"],
                  "kernel_us": result["kernel_us"], "copy_ceiling_GBps": result["copy_ceiling"]["GBps"],
                  "roofline": result["roofline"]}
    ctx.close()
    return result


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", choices=["all", "c0", "c1", "c2", "c3", "c3_hot", "c4"], default="all",
                    help="all (default): C1 in full as the headline, then C0, C2, C3, the C3 stress point and C4 "
                         "briefly, as per-configuration blocks of the same JSON line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--brief", action="store_true",
                    help="with --workload cN: the configuration's block as the default run prints it (no variants)")
    ap.add_argument("--schedule", choices=["auto", "aligned", "pipelined", "one_stream", "one_launch", "launch_and_plan", "free", "single"], default="auto",
                    help="how the send side and the receive side of a step are issued (see step())")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--row-stride", type=int, default=None,
                    help="bytes from row to row in packed / received arrays (default: row bytes rounded up to 128)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the other ranks of the dispatch are "
              "simulated); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.workload == "all":
        result = bench_dispatch(args, "c1")
        configs = {"C1": {k: result[k] for k in ("steps", "warmup", "ms_per_step", "pct_of_hbm_peak",
                                                 "bytes_saved_vs_unicast", "roofline")}}
        configs["C1"].update(GBps=result["value"], schedule=result["config"]["schedule"])
        import copy
        import gc
        args_b = copy.copy(args)          # the brief blocks time at least 100 steps each: at 0.1 ms a step the
        args_b.steps = max(args.steps, 100)       # start and the end of a shorter timed region weigh over 1 %
        args_b.warmup = max(args.warmup, 10)
        for name in ("c0", "c2", "c3", "c3_hot", "c4"):
            gc.collect()
            torch.cuda.empty_cache()
            t0 = time.time()
            configs[name.upper()] = (bench_allgather(args_b, brief=True) if name == "c4"
                                     else bench_dispatch(args_b, name, brief=True))
            log("[bench] %s done in %.1fs" % (name, time.time() - t0))
        result["configs"] = {k: configs[k] for k in sorted(configs)}
        result["configs_note"] = ("C0 and the 4 MiB pack of C4 are launch-latency bound: their percentages of the HBM "
                                  "peak are not meaningful; C3_HOT is the skew stress point of C3 (hottest rank, 512 "
                                  "tokens per peer)")
    else:
        result = (bench_allgather(args, args.brief) if args.workload == "c4"
                  else bench_dispatch(args, args.workload, args.brief))
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
