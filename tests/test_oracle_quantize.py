"""Pins of the oracle's block-wise fp8 quantiser (quantise-in-pack contract) against a
hand-worked block, a library conversion (PyTorch's CPU cast to float8_e4m3fn), a brute-force
nearest-value search in exact rational arithmetic, and the properties the contract implies.
CPU only."""
import json
import os
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2605_22428_amd import workloads as W


def bf16_bits(v) -> np.ndarray:
    """float32 values that are exactly representable in bf16 -> their bit patterns."""
    a = np.ascontiguousarray(v, dtype=np.float32)
    bits = a.view(np.uint32)
    assert not (bits & 0xffff).any(), "value is not a bf16 number"
    return (bits >> 16).astype(np.uint16)


def bf16_value(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def decode(code: int) -> Fraction:
    """Value of a finite e4m3 code, from the format definition, exactly."""
    sign = -1 if code & 0x80 else 1
    e, m = (code >> 3) & 15, code & 7
    mag = Fraction(m, 512) if e == 0 else Fraction(8 + m) * Fraction(2) ** (e - 10)
    return sign * mag


FINITE = [c for c in range(256) if (c & 0x7f) != 0x7f]


def block_of(values, fill=0.0):
    row = np.full(128, fill, dtype=np.float32)
    row[: len(values)] = values
    return bf16_bits(row)[None, :]


def test_hand_worked_block(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "e4m3_block_example.json")))
    codes, scales = ref.quantize_rows(block_of(g["values"]))
    assert [format(int(c), "02x") for c in codes[0, : len(g["values"])]] == g["codes_hex"]
    assert float(scales[0, 0]) == g["scale"]
    assert not codes[0, len(g["values"]):].any()


@pytest.mark.parametrize("k", [-12, -3, 0, 5, 40])
def test_every_code_survives_a_round_trip_and_ties_go_to_even(k):
    """With a block maximum of 448 * 2^k the scale is exactly 2^k, so x = value(code) * 2^k must
    come back as that code, and exact midpoints must go to the even neighbour."""
    pos = [c for c in FINITE if c < 0x80]
    vals = [float(decode(c)) * 2.0 ** k for c in pos] + [-float(decode(c)) * 2.0 ** k for c in pos]
    for lo in range(0, len(vals), 127):
        chunk = vals[lo:lo + 127]
        codes, scales = ref.quantize_rows(block_of([448.0 * 2.0 ** k] + chunk))
        assert float(scales[0, 0]) == 2.0 ** k
        want = [0x7e] + [(c if v >= 0 and not (v == 0 and np.signbit(v)) else c | 0x80)
                         for v, c in zip(chunk, (pos + pos)[lo:lo + 127])]
        got = codes[0, : len(chunk) + 1].tolist()
        # -0.0 carries its sign
        want = [w if not (w == 0 and np.signbit(np.float32(v))) else 0x80
                for w, v in zip(want, [448.0] + chunk)]
        assert got == want
    mids = [(decode(c) + decode(c + 1)) / 2 for c in range(0, 126)]
    even = [c if c % 2 == 0 else c + 1 for c in range(0, 126)]
    codes, _ = ref.quantize_rows(block_of([448.0 * 2.0 ** k] + [float(m) * 2.0 ** k for m in mids]))
    assert codes[0, 1:127].tolist() == even
    codes, _ = ref.quantize_rows(block_of([448.0 * 2.0 ** k] + [-float(m) * 2.0 ** k for m in mids]))
    assert codes[0, 1:127].tolist() == [c | 0x80 for c in even]


def _recompute_y(x_bits, scales):
    """The contract's y = x * (448 / a_c) in numpy float32 (IEEE, one rounding per operation)."""
    x = bf16_value(x_bits).reshape(x_bits.shape[0], -1, 128)
    a = np.abs(x).max(axis=2)
    a_c = np.maximum(a, np.float32(2.0 ** -20)).astype(np.float32)
    s = (a_c / np.float32(448.0)).astype(np.float32)
    inv = (np.float32(448.0) / a_c).astype(np.float32)
    y = np.clip((x * inv[:, :, None]).astype(np.float32), np.float32(-448.0), np.float32(448.0))
    assert s.tobytes() == scales.tobytes()
    return y.reshape(x_bits.shape[0], -1), s


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_against_the_library_cast_and_a_brute_force_search(seed):
    w = W.DispatchWorkload("q", 51, 8, 16, 2, 40, 1024, "bf16", "uniform")
    x_bits, _ = W.payload_rows(w, seed, 0)
    # widen the dynamic range: some blocks tiny, some huge, some with exact zeros and negatives
    x = bf16_value(x_bits).copy()
    x[3] *= np.float32(2.0 ** -30); x[4] *= np.float32(2.0 ** 60); x[5, 100:300] = 0.0; x[6] = 0.0
    x[7, ::2] = -np.abs(x[7, ::2])
    x_bits = W.f32_to_bf16_bits(x)
    codes, scales = ref.quantize_rows(x_bits)
    y, s = _recompute_y(x_bits, scales)
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert codes.tobytes() == lib.tobytes()
    # brute force: nearest finite value over all codes, exact arithmetic, ties to the even code
    rng = np.random.default_rng(seed)
    table = [(decode(c), c) for c in FINITE if c < 0x80]
    for r, j in zip(rng.integers(0, x.shape[0], 300), rng.integers(0, x.shape[1], 300)):
        yy = Fraction(float(abs(y[r, j])))
        best = min(table, key=lambda vc: (abs(vc[0] - yy), vc[1] & 1))
        assert (int(codes[r, j]) & 0x7f) == best[1], (r, j, float(yy))
        assert (int(codes[r, j]) >> 7) == int(np.signbit(y[r, j]))


def test_scale_maximum_and_error_bound():
    w = W.DispatchWorkload("q", 52, 8, 16, 2, 64, 512, "bf16", "uniform")
    x_bits, _ = W.payload_rows(w, 9, 1)
    codes, scales = ref.quantize_rows(x_bits)
    x = bf16_value(x_bits).astype(np.float64).reshape(64, 4, 128)
    a = np.abs(x).max(axis=2)
    assert np.all(np.abs(scales.astype(np.float64) * 448.0 - a) <= a * 2.0 ** -23)
    c = codes.reshape(64, 4, 128)
    # the block maximum maps to +-448
    top = np.abs(x) == a[:, :, None]
    assert np.all((c[top] & 0x7f) == 0x7e)
    # dequantised values: within half a step of the format at that magnitude (relative 2^-4 for
    # normal numbers, absolute 2^-10 * scale below the smallest normal), plus rounding slack
    val = np.array([float(decode(int(v))) for v in c.reshape(-1)]).reshape(c.shape)
    deq = val * scales.astype(np.float64)[:, :, None]
    bound = np.maximum(np.abs(x) * 2.0 ** -4, scales.astype(np.float64)[:, :, None] * 2.0 ** -10) * (1 + 2.0 ** -20)
    assert np.all(np.abs(deq - x) <= bound)
    # monotone inside a block: larger input never gets a smaller value
    for r, b in ((0, 0), (10, 3), (63, 1)):
        order = np.argsort(x[r, b], kind="stable")
        assert np.all(np.diff(val[r, b][order]) >= 0)


def test_all_zero_block_and_refused_inputs():
    codes, scales = ref.quantize_rows(np.zeros((2, 256), np.uint16))
    assert not codes.any() and np.all(scales == np.float32(2.0 ** -20) / np.float32(448.0))
    neg0 = np.full((1, 128), 0x8000, np.uint16)
    codes, _ = ref.quantize_rows(neg0)
    assert np.all(codes == 0x80)
    for pattern in (0x7f80, 0xff80, 0x7fc0):          # +inf, -inf, NaN
        bad = np.zeros((1, 128), np.uint16); bad[0, 5] = pattern
        with pytest.raises(ref.OracleError):
            ref.quantize_rows(bad)
    with pytest.raises(ref.OracleError):
        ref.quantize_rows(np.zeros((1, 100), np.uint16))
