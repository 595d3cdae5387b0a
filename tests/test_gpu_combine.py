"""GPU parity of mw_combine_gather (the way back: one returned row per received row, the
single-precision sum of its local experts' outputs) against the CPU oracle.  Both sides add
the same bf16 values in the same order in single precision and round once, so the bar is
bit-exact."""
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


def bf16_value(bits):
    return (np.asarray(bits).astype(np.uint32) << 16).view(np.float32)


def run_combine(w, seed, my_rank, lazy=False, y_kind="normal", edit=None, packets=False):
    _say("combine", w.name, "seed", seed, "my_rank", my_rank, "T", w.n_tokens, "H", w.hidden, y_kind)
    e2r = W.expert_to_rank(w)
    ctx = H.make_ctx(w, my_rank)
    topks = W.topk_ids_many(w, seed, range(w.n_ranks))
    x_dev = torch.zeros((w.n_tokens, w.hidden), dtype=torch.int16, device=H.DEV) if lazy else None
    recs, bufs, toks, pk = [], [], [], []
    for p in range(w.n_ranks):
        tk = topks[p]
        if edit is not None:
            edit(p, tk)
        if lazy:
            tokens = W.tokens_for_rank(w, tk, my_rank)
            rows, _ = W.payload_rows(w, seed, p, tokens)
            x = np.zeros((w.n_tokens, w.hidden), dtype=rows.dtype)
            x[tokens] = rows
            x_dev.zero_()
            x_dev[torch.from_numpy(tokens).to(H.DEV)] = H.dev(rows).view(torch.int16)
            g = H.GpuSend(ctx, tk, x, None, x_dev=x_dev)
        else:
            x, _ = W.payload_rows(w, seed, p)
            g = H.GpuSend(ctx, tk, x, None)
        _, perm, desc, _ = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
        packed, src, rtk = ref.pack(x, None, tk, perm)
        bufs.append(ref.deliver(desc, packed, src, rtk, my_rank))
        toks.append((tk, x, None))
        recs.append(H.shrink(g.deliver(my_rank)))
        del g
    m_rows = sum(r["n_rows"] for r in recs)
    cap = max(1, m_rows * min(w.top_k, w.experts_per_rank))
    plain = ref.dispatch_plain(toks, e2r, my_rank, cap)
    gu = H.GpuUnpack(ctx, recs, cap)
    H.check_unpack(gu, plain, "dispatch before the way back")
    Q = gu.Q
    rng = np.random.default_rng(seed + 17)
    if y_kind == "identity":
        y_bits = plain[0].view(np.uint16).reshape(Q, w.hidden).copy()
    elif y_kind == "ints":
        y_bits = W.f32_to_bf16_bits(rng.integers(-3, 4, size=(Q, w.hidden)).astype(np.float32))
    else:
        y = rng.standard_normal((Q, w.hidden), dtype=np.float32) * np.float32(3.0)
        y[::7] *= np.float32(2.0 ** 20); y[3::11] *= np.float32(2.0 ** -30)
        y_bits = W.f32_to_bf16_bits(y)
    y_dev = torch.zeros((cap, w.hidden), dtype=torch.int16, device=H.DEV)
    y_dev[:Q] = H.dev(y_bits)
    ret = torch.zeros((max(m_rows, 1), w.hidden), dtype=torch.int16, device=H.DEV)
    ctx.mw_combine_gather(len(recs), y_dev, cap, ret, m_rows)
    torch.cuda.synchronize()
    want = ref.combine_gather(bufs, w.top_k, e2r, my_rank, y_bits, plain[2], plain[3], plain[4])
    want = np.concatenate(want) if want else np.zeros((0, w.hidden), np.uint16)
    got = H.host(ret).view(np.uint16)[:m_rows]
    H.assert_same_bytes(got, want, "returned rows")
    if y_kind == "ints":
        assert np.array_equal(bf16_value(got).astype(np.float64).sum(axis=0),
                              bf16_value(y_bits).astype(np.float64).sum(axis=0))
    multi = sum(1 for b in bufs for _ in b[2]) and (Q - m_rows)
    _say("  rows back", m_rows, "expert outputs", Q, "extra hits folded", multi)
    ctx.close()
    return got, want


@pytest.mark.parametrize("seed", [W.BASE_SEED, 1])
@pytest.mark.parametrize("y_kind", ["normal", "ints", "identity"])
def test_c0_tiny(seed, y_kind):
    run_combine(W.C0, seed, 5, y_kind=y_kind)


@pytest.mark.parametrize("seed", [1, 2])
def test_c1_shape_reduced(seed):
    run_combine(W.scaled(W.C1, n_tokens=333, hidden=1024), seed, 37)


def test_many_local_experts_per_token():
    # 4 ranks x 8 experts, top-6: most tokens reach several experts of one rank
    def edit(p, tk):
        tk[p % 3::5, 2] = tk[p % 3::5, 0]
        tk[1::7, 4] = -1
    w = W.DispatchWorkload("dense", 71, 4, 32, 6, 150, 512, "bf16", "uniform")
    run_combine(w, 3, 2, edit=edit)
    run_combine(w, 4, 0, y_kind="ints", edit=edit)


def test_more_than_eight_local_experts_per_row():
    run_combine(W.DispatchWorkload("dense20", 91, 2, 40, 24, 100, 256, "bf16", "uniform"), 1, 1)
    run_combine(W.DispatchWorkload("k64", 92, 4, 128, 64, 60, 128, "bf16", "uniform"), 2, 3, y_kind="ints")


def test_full_width_rows():
    run_combine(W.DispatchWorkload("wide_bf16", 11, 8, 16, 2, 257, 7168, "bf16", "uniform"), 1, 3)


def test_c1_full_size():
    run_combine(W.C1, W.BASE_SEED, 0, lazy=True)


def test_refused_for_other_row_formats_and_bounded_by_capacity():
    w8 = W.DispatchWorkload("small_fp8", 12, 8, 16, 2, 16, 512, "fp8", "uniform")
    ctx = H.make_ctx(w8, 0)
    buf = torch.zeros((16, 512), dtype=torch.int16, device=H.DEV)
    with pytest.raises(B.MwError) as ei:
        ctx.mw_combine_gather(8, buf, 16, buf, 16)
    assert ei.value.status == B.MW_ERR_UNSUPPORTED
    ctx.close()
    # a return buffer shorter than the rows received: the rest is simply not written
    w = W.DispatchWorkload("small", 31, 8, 16, 2, 64, 256, "bf16", "uniform")
    e2r = W.expert_to_rank(w)
    ctx = H.make_ctx(w, 1)
    recs, bufs, toks = [], [], []
    for p in range(w.n_ranks):
        tk = W.topk_ids(w, 2, p); x, _ = W.payload_rows(w, 2, p)
        g = H.GpuSend(ctx, tk, x, None)
        recs.append(H.shrink(g.deliver(1)))
        _, perm, desc, _ = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
        packed, src, rtk = ref.pack(x, None, tk, perm)
        bufs.append(ref.deliver(desc, packed, src, rtk, 1)); toks.append((tk, x, None))
    m = sum(r["n_rows"] for r in recs)
    plain = ref.dispatch_plain(toks, e2r, 1, 2 * m)
    gu = H.GpuUnpack(ctx, recs, 2 * m)
    y_bits = plain[0].view(np.uint16).reshape(gu.Q, w.hidden)
    y_dev = torch.zeros((2 * m, w.hidden), dtype=torch.int16, device=H.DEV)
    y_dev[: gu.Q] = H.dev(y_bits)
    ret = torch.full((m, w.hidden), 0x1234, dtype=torch.int16, device=H.DEV)
    short = m // 2
    ctx.mw_combine_gather(len(recs), y_dev, 2 * m, ret, short)
    torch.cuda.synchronize()
    want = np.concatenate(ref.combine_gather(bufs, w.top_k, e2r, 1, y_bits, plain[2], plain[3], plain[4]))
    got = H.host(ret).view(np.uint16)
    H.assert_same_bytes(got[:short], want[:short], "rows below the return capacity")
    assert np.all(got[short:] == 0x1234)
    ctx.close()
