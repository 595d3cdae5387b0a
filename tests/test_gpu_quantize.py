"""GPU parity of mw_pack_quantize (bf16 rows quantised to fp8 rows inside the packer) against
the CPU oracle's quantiser followed by its packer.  Every code is an integer decision taken
from single-precision arithmetic on both sides; the bar is bit-exact codes and scales."""
import dataclasses

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
    return (bits.astype(np.uint32) << 16).view(np.float32)


def gpu_pack_quantize(ctx, tk, x_bits):
    T = tk.shape[0]
    tk_d, x_d = H.dev(tk.astype(np.int32)), H.dev(x_bits)
    buf = B.SendBuffers(ctx, T)
    ctx.mw_plan(tk_d, buf.mask, buf.perm, buf.desc, buf.stats)
    ctx.mw_pack_quantize(x_d, tk_d, buf.perm, buf.stats, buf.packed, buf.row_src_token, buf.row_topk)
    st = ctx.mw_get_send_stats(buf.stats)
    n = int(st["n_rows"])
    whole = H.host(buf.packed)[:n]
    assert not whole[:, ctx.row_bytes:].any(), "bytes between packed rows were written"
    return whole[:, : ctx.row_bytes], H.host(buf.row_src_token)[:n], H.host(buf.row_topk)[:n], H.host(buf.perm)[:n]


def check(w_fp8, tk, x_bits, rows=None, row_stride=0):
    """rows: check only these packed rows against the oracle (full sizes); None = all."""
    e2r = W.expert_to_rank(w_fp8)
    ctx = H.make_ctx(w_fp8, 0, max_recv_rows=1, max_tokens=max(tk.shape[0], 1), row_stride=row_stride)
    packed, src, rtk, perm_g = gpu_pack_quantize(ctx, tk, x_bits)
    _, perm, _, _ = ref.plan(tk, e2r, w_fp8.n_ranks, w_fp8.row_bytes)
    H.assert_same_bytes(perm_g, perm, "perm")
    H.assert_same_bytes(src, perm, "row_src_token")
    H.assert_same_bytes(rtk, tk[perm], "row_topk")
    pick = np.arange(len(perm)) if rows is None else np.asarray(rows)
    codes, scales = ref.quantize_rows(x_bits[perm[pick]])
    want = np.concatenate([codes, scales.view(np.uint8).reshape(len(pick), -1)], axis=1)
    got = packed[pick]
    if got.tobytes() != want.tobytes():
        bad = np.argwhere(got != want)
        r, c = bad[0]
        raise AssertionError("%d differing bytes; first: packed row %d byte %d (H=%d) got %#x want %#x, input %r"
                             % (len(bad), pick[r], c, w_fp8.hidden, got[r, c], want[r, c],
                                float(bf16_value(x_bits[perm[pick[r]]])[min(c, w_fp8.hidden - 1)])))
    ctx.close()
    return packed


def _inputs(w_fp8, seed, wide_range=True):
    w_bf = dataclasses.replace(w_fp8, row_format="bf16")      # same values, before quantisation
    tk = W.topk_ids(w_fp8, seed, 0)
    x_bits, _ = W.payload_rows(w_bf, seed, 0)
    if wide_range:
        x = bf16_value(x_bits).copy()
        n = x.shape[0]
        x[3 % n] *= np.float32(2.0 ** -30); x[4 % n] *= np.float32(2.0 ** 60)
        x[5 % n, 100:300] = 0.0; x[6 % n] = 0.0
        x[7 % n, ::2] = -np.abs(x[7 % n, ::2])
        x[8 % n] *= np.float32(2.0 ** -125)                      # subnormal bf16 inputs
        x_bits = W.f32_to_bf16_bits(x)
        x_bits[9 % n, :64] = 0x8000                                # negative zeros
    return tk, x_bits


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_c2_shape_reduced(seed):
    w = W.scaled(W.C2, n_tokens=333, hidden=1024)
    _say("quantize", w.name, seed)
    tk, x_bits = _inputs(w, seed)
    check(w, tk, x_bits)


def test_full_width_rows_ragged_token_count():
    w = W.DispatchWorkload("wide_fp8", 12, 8, 16, 2, 129, 7168, "fp8", "uniform")
    tk, x_bits = _inputs(w, 5)
    tk[11] = -1                       # a token that goes nowhere is not packed
    check(w, tk, x_bits)
    w = W.DispatchWorkload("narrow_fp8", 13, 8, 16, 2, 40, 512, "fp8", "uniform")
    check(w, *_inputs(w, 6))
    check(w, *_inputs(w, 7), row_stride=640)              # rows of 528 bytes, 640 apart


def test_every_code_and_every_exact_tie():
    """Blocks whose maximum is 448 * 2^k have scale 2^k exactly: inputs value(code) * 2^k must
    come back as that code and exact midpoints must go to the even neighbour -- this is the
    hardware conversion's rounding, checked on all 254 finite codes."""
    w = W.DispatchWorkload("codes_fp8", 14, 8, 16, 2, 16, 512, "fp8", "uniform")
    tk = W.topk_ids(w, 1, 0)
    dec = lambda c: ((c & 7) * 2.0 ** -9) if (c >> 3) == 0 else (8 + (c & 7)) * 2.0 ** ((c >> 3) - 10)
    pos = [dec(c) for c in range(127)]
    mids = [(pos[c] + pos[c + 1]) / 2 for c in range(126)]
    x = np.zeros((w.n_tokens, w.hidden), dtype=np.float32)
    for r, k in enumerate((-12, -3, 0, 5)):
        sgn = 1.0
        for half in range(2):
            row = 4 * half + r
            x[row, 0:127] = np.array(pos) * 2.0 ** k * sgn;  x[row, 127] = 448.0 * 2.0 ** k
            x[row, 128:254] = np.array(mids) * 2.0 ** k * sgn; x[row, 255] = 448.0 * 2.0 ** k
            sgn = -1.0
    x_bits = W.f32_to_bf16_bits(x)
    assert np.array_equal(bf16_value(x_bits), x)         # all inputs are bf16 numbers
    packed = check(w, tk, x_bits)
    assert packed.shape[0] == w.n_tokens


def test_c2_full_size_sampled_rows():
    w = W.C2
    _say("quantize full size", w.name)
    tk, x_bits = _inputs(w, W.BASE_SEED)
    n = int((tk != -1).any(axis=1).sum())
    check(w, tk, x_bits, rows=np.arange(0, n, 13))


def test_wrong_row_format_is_refused():
    w = W.DispatchWorkload("small", 31, 8, 16, 2, 16, 512, "bf16", "uniform")
    ctx = H.make_ctx(w, 0)
    tk = H.dev(W.topk_ids(w, 1, 0))
    buf = B.SendBuffers(ctx, w.n_tokens)
    ctx.mw_plan(tk, buf.mask, buf.perm, buf.desc, buf.stats)
    x = torch.zeros((w.n_tokens, w.hidden), dtype=torch.int16, device=H.DEV)
    with pytest.raises(B.MwError) as ei:
        ctx.mw_pack_quantize(x, tk, buf.perm, buf.stats, buf.packed, buf.row_src_token, buf.row_topk)
    assert ei.value.status == B.MW_ERR_UNSUPPORTED
    ctx.close()
