"""Pins of the oracle's way-back step (ref_combine_gather: one row per received row, the sum
of its local experts' outputs) against closed forms, a brute-force summation written
separately in Python, exact integer conservation and a hand-worked case where the order of
summation decides the result.  CPU only."""
import numpy as np
import pytest

from oracle import ref
from paper_2605_22428_amd import workloads as W

import brute


def bf16_value(bits):
    return (np.asarray(bits).astype(np.uint32) << 16).view(np.float32)


def _setup(w, seed, my_rank, edit=None):
    e2r = W.expert_to_rank(w)
    toks, bufs = [], []
    for p in range(w.n_ranks):
        tk = W.topk_ids(w, seed, p)
        if edit is not None:
            edit(p, tk)
        x, _ = W.payload_rows(w, seed, p)
        _, perm, desc, _ = ref.plan(tk, e2r, w.n_ranks, w.row_bytes)
        packed, src, rtk = ref.pack(x, None, tk, perm)
        toks.append((tk, x, None))
        bufs.append(ref.deliver(desc, packed, src, rtk, my_rank))
    plain = ref.dispatch_plain(toks, e2r, my_rank, 10 ** 5)
    return e2r, toks, bufs, plain


def _hits(e2r, my_rank, ids):
    """distinct local experts of a token, in the order of its id list"""
    out = []
    for e in ids:
        if e != -1 and e2r[e] == my_rank and e not in out:
            out.append(int(e))
    return out


def _brute(e2r, my_rank, toks, bufs, plain, y_bits):
    """Separate derivation: position lookup from the plain definition's (peer, token) lists,
    sequential numpy float32 additions, the generator's bf16 rounding."""
    _, _, sp, stok, offs = plain
    local = [e for e in range(len(e2r)) if e2r[e] == my_rank]
    where = {}
    for le, e in enumerate(local):
        for q in range(int(offs[le]), int(offs[le + 1])):
            where[(e, int(sp[q]), int(stok[q]))] = q
    y = bf16_value(y_bits)
    outs = []
    for p, (desc, rows, src, rtk) in enumerate(bufs):
        out = np.zeros((len(src), y.shape[1]), dtype=np.uint16)
        for i, t in enumerate(src):
            hs = _hits(e2r, my_rank, toks[p][0][t])
            assert hs, "a delivered row has a local expert"
            if len(hs) == 1:
                out[i] = y_bits[where[(hs[0], p, int(t))]]
                continue
            acc = y[where[(hs[0], p, int(t))]].copy()
            for e in hs[1:]:
                acc = (acc + y[where[(e, p, int(t))]]).astype(np.float32)
            out[i] = W.f32_to_bf16_bits(acc)
        outs.append(out)
    return outs


@pytest.mark.parametrize("seed,my_rank", [(1, 0), (2, 3)])
def test_identity_experts_give_h_times_the_token(seed, my_rank):
    """If every expert returns its input, a token that reached h local experts comes back as
    h * x rounded once to bf16 (h * x is exact in single precision for h <= 8)."""
    w = W.DispatchWorkload("t", 61, 4, 16, 4, 50, 256, "bf16", "uniform")     # 4 experts per rank
    e2r, toks, bufs, plain = _setup(w, seed, my_rank)
    y_bits = plain[0].view(np.uint16).reshape(len(plain[2]), w.hidden)
    ret = ref.combine_gather(bufs, w.top_k, e2r, my_rank, y_bits, plain[2], plain[3], plain[4])
    seen_h = set()
    for p, (desc, rows, src, rtk) in enumerate(bufs):
        assert ret[p].shape == (len(src), w.hidden)
        for i, t in enumerate(src):
            h = len(_hits(e2r, my_rank, toks[p][0][t]))
            seen_h.add(h)
            x = bf16_value(toks[p][1][t]).astype(np.float64)
            want = toks[p][1][t] if h == 1 else W.f32_to_bf16_bits((h * x).astype(np.float32))
            assert ret[p][i].tobytes() == np.asarray(want).tobytes(), (p, i, h)
    assert {1, 2, 3} <= seen_h


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_against_a_separate_summation_and_the_exact_sum(seed):
    w = W.DispatchWorkload("t", 62, 6, 30, 5, 40, 128, "bf16", "uniform")
    my_rank = seed % w.n_ranks

    def edit(p, tk):
        tk[p % 4::6, 2] = -1
        tk[(p + 1) % 5::5, 1] = tk[(p + 1) % 5::5, 0]
    e2r, toks, bufs, plain = _setup(w, seed, my_rank, edit)
    Q = len(plain[2])
    rng = np.random.default_rng(seed)
    y_bits = W.f32_to_bf16_bits((rng.standard_normal((Q, w.hidden)) * 3.0).astype(np.float32))
    ret = ref.combine_gather(bufs, w.top_k, e2r, my_rank, y_bits, plain[2], plain[3], plain[4])
    want = _brute(e2r, my_rank, toks, bufs, plain, y_bits)
    for p in range(w.n_ranks):
        assert ret[p].tobytes() == want[p].tobytes(), p
    # and within one bf16 step of the exact sum
    y64 = bf16_value(y_bits).astype(np.float64)
    _, _, sp, stok, offs = plain
    total = np.zeros(w.hidden)
    for p, (desc, rows, src, rtk) in enumerate(bufs):
        for i, t in enumerate(src):
            qs = [q for q in range(Q) if sp[q] == p and stok[q] == t]
            exact = y64[qs].sum(axis=0)
            got = bf16_value(ret[p][i]).astype(np.float64)
            assert np.all(np.abs(got - exact) <= np.maximum(np.abs(exact), 2.0 ** -120) * 2.0 ** -7)


def test_small_integers_are_conserved_exactly():
    """Every expert output row contributes to exactly one returned row: with small integer
    values all sums are exact, so the totals must agree exactly."""
    w = W.DispatchWorkload("t", 63, 4, 12, 3, 64, 64, "bf16", "uniform")
    my_rank = 2
    e2r, toks, bufs, plain = _setup(w, 5, my_rank)
    Q = len(plain[2])
    rng = np.random.default_rng(5)
    y = rng.integers(-3, 4, size=(Q, w.hidden)).astype(np.float32)
    y_bits = W.f32_to_bf16_bits(y)
    ret = ref.combine_gather(bufs, w.top_k, e2r, my_rank, y_bits, plain[2], plain[3], plain[4])
    total = sum(bf16_value(r).astype(np.float64).sum(axis=0) for r in ret)
    assert np.array_equal(total, y.astype(np.float64).sum(axis=0))
    assert sum(len(r) for r in ret) == plain_rows(bufs)


def plain_rows(bufs):
    return sum(len(b[2]) for b in bufs)


def test_the_order_of_the_id_list_is_the_order_of_summation():
    """Hand-worked: a = 2^16, b = 256, c = d = 0.75 * 2^-8.  In single precision
    ((a + b) + c) + d = 2^16 + 256 (c and d are each below half a unit in the last place and
    vanish), a tie for bf16 that goes to the even 2^16 = 0x4780; ((c + d) + a) + b =
    2^16 + 256 + 2^-7, above the tie, so bf16 gives 2^16 + 512 = 0x4781."""
    e2r = np.zeros(4, dtype=np.int32)                     # one rank hosting experts 0..3
    tk = np.array([[0, 1, 2, 3], [2, 3, 0, 1], [1, -1, -1, -1]], dtype=np.int32)
    x = np.zeros((3, 8), dtype=np.uint16)
    _, perm, desc, _ = ref.plan(tk, e2r, 1, 16)
    packed, src, rtk = ref.pack(x, None, tk, perm)
    bufs = [ref.deliver(desc, packed, src, rtk, 0)]
    plain = ref.dispatch_plain([(tk, x, None)], e2r, 0, 100)
    vals = {0: 2.0 ** 16, 1: 256.0, 2: 0.75 * 2.0 ** -8, 3: 0.75 * 2.0 ** -8}
    offs = plain[4]
    y = np.zeros((len(plain[2]), 8), dtype=np.float32)
    for e in range(4):
        y[int(offs[e]):int(offs[e + 1])] = vals[e]
    y_bits = W.f32_to_bf16_bits(y)
    assert np.array_equal(bf16_value(y_bits), y)
    ret = ref.combine_gather(bufs, 4, e2r, 0, y_bits, plain[2], plain[3], plain[4])[0]
    by_token = {int(t): ret[i] for i, t in enumerate(src)}
    assert set(by_token[0].tolist()) == {0x4780}
    assert set(by_token[1].tolist()) == {0x4781}
    assert by_token[2].tobytes() == y_bits[int(offs[1]) + [int(v) for v in plain[3][int(offs[1]):int(offs[2])]].index(2)].tobytes()


def test_inconsistent_layout_is_refused():
    w = W.DispatchWorkload("t", 64, 4, 8, 2, 20, 32, "bf16", "uniform")
    e2r, toks, bufs, plain = _setup(w, 1, 1)
    y_bits = np.zeros((len(plain[2]), w.hidden), np.uint16)
    stok = plain[3].copy(); stok[0] = 10 ** 6              # the layout no longer holds that token
    with pytest.raises(ref.OracleError):
        ref.combine_gather(bufs, w.top_k, e2r, 1, y_bits, plain[2], stok, plain[4])
