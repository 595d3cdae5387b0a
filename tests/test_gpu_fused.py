"""GPU parity of mw_plan_pack (plan and pack of a decode-sized batch in one launch) against
the CPU oracle's plan and pack, bit-exact, and against the two-call path's buffers."""
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


def _one(w, seed, rank, edit=None, row_stride=0):
    _say("fused", w.name, "seed", seed, "rank", rank, "T", w.n_tokens, "H", w.hidden, w.row_format)
    tk = W.topk_ids(w, seed, rank)
    if edit is not None:
        edit(tk)
    x, sc = W.payload_rows(w, seed, rank)
    ctx = H.make_ctx(w, rank, max_recv_rows=1, row_stride=row_stride)
    g = H.GpuSend(ctx, tk, x, sc, fused=True)
    H.check_send(w, g, tk, x, sc)
    two = H.GpuSend(ctx, tk, x, sc)                      # the two-call path, whole buffers
    for name in ("mask", "perm", "desc", "stats", "packed", "row_src_token", "row_topk"):
        H.assert_same_bytes(H.host(getattr(g.buf, name)), H.host(getattr(two.buf, name)), "fused vs two calls: " + name)
    ctx.close()
    return g


@pytest.mark.parametrize("seed", [W.BASE_SEED, 1, 2])
def test_c0_whole_batch(seed):
    _one(W.C0, seed, 3)


@pytest.mark.parametrize("T", [1, 63, 64, 65, 128, 255, 256])
def test_c1_shape_decode_batches(T):
    _one(W.scaled(W.C1, n_tokens=T, hidden=1024), 5, 17)


@pytest.mark.parametrize("T", [64, 200])
def test_wide_bitmaps(T):
    # 256 ranks: four bitmap words
    _one(W.scaled(W.C3, n_tokens=T, hidden=512), 1, 100)
    # 128 ranks: two words
    _one(W.DispatchWorkload("r128", 21, 128, 256, 6, T, 256, "bf16", "uniform"), 2, 77)
    # twelve ids per token: more bits than a short key holds, whole bitmaps are compared
    _one(W.DispatchWorkload("k12", 22, 256, 512, 12, T, 256, "bf16", "uniform"), 3, 200)
    _one(W.DispatchWorkload("k9", 23, 192, 192, 9, T, 256, "bf16", "uniform"), 4, 5)


def test_full_width_rows_bf16_and_fp8():
    _one(W.scaled(W.C2, n_tokens=100, hidden=1024), 6, 3, row_stride=1152)      # rows of 1056 bytes, 1152 apart
    _one(W.scaled(W.C1, n_tokens=128), W.BASE_SEED, 0)
    _one(W.scaled(W.C2, n_tokens=64), W.BASE_SEED, 9)
    _one(W.scaled(W.C2, n_tokens=129, hidden=1024), 4, 9)


def test_empty_tokens_duplicates_and_few_groups():
    w = W.DispatchWorkload("small", 31, 8, 16, 4, 96, 256, "bf16", "uniform")

    def edit(tk):
        tk[::3, 1] = tk[::3, 0]
        tk[1::5, 3] = -1
        tk[7] = -1
        tk[95] = -1
    _one(w, 8, 2, edit)

    def same(tk):
        tk[:] = np.array([5, 0, 5, -1], dtype=np.int32)
    g = _one(w, 8, 2, same)
    assert g.G == 1 and g.N == 96

    def none(tk):
        tk[:] = -1
    g = _one(w, 8, 2, none)
    assert (g.N, g.G, int(g.stats["unicast_bytes"])) == (0, 0, 0)


def test_empty_batch_bad_ids_and_capacity():
    w = W.DispatchWorkload("small", 31, 8, 16, 2, 128, 256, "bf16", "uniform")
    ctx = H.make_ctx(w, 0, max_tokens=512)
    g = H.GpuSend(ctx, np.zeros((0, 2), np.int32), np.zeros((0, w.hidden), np.uint16), None, fused=True)
    assert (g.N, g.G, int(g.stats["unicast_bytes"]), int(g.stats["error_flags"])) == (0, 0, 0, 0)
    assert int(H.host(g.buf.perm)[0]) == -1              # untouched
    tk = W.topk_ids(w, 1, 0)
    x, _ = W.payload_rows(w, 1, 0)
    bad = tk.copy(); bad[7, 1] = w.n_experts; bad[20, 0] = -5
    g = H.GpuSend(ctx, bad, x, None, fused=True)
    assert int(g.stats["error_flags"]) == B.MW_FLAG_BAD_EXPERT
    ign = bad.copy(); ign[7, 1] = -1; ign[20, 0] = -1
    m, perm, desc, st = ref.plan(ign, W.expert_to_rank(w), w.n_ranks, w.row_bytes)
    H.assert_same_bytes(g.host_plan()[1], perm, "perm with ignored ids")
    H.assert_same_bytes(g.host_plan()[2].view(np.uint8), desc.view(np.uint8), "desc with ignored ids")
    g = H.GpuSend(ctx, tk, x, None, fused=True)
    assert int(g.stats["error_flags"]) == 0              # the flag does not stick
    # more tokens than one launch takes: refused on the host, nothing written
    big = np.zeros((B.MW_FUSED_MAX_TOKENS + 1, 2), np.int32)
    with pytest.raises(B.MwError) as ei:
        H.GpuSend(ctx, big, np.zeros((len(big), w.hidden), np.uint16), None, fused=True)
    assert ei.value.status == B.MW_ERR_CAPACITY
    ctx.close()
