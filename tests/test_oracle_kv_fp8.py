"""Pins of the oracle's 8-bit slot format (oracle/kv_fp8.py) against the format's definition and a library routine.

The element code is E4M3 of the OCP 8-bit floating point specification; nothing here comes from the HIP path."""
import math

import numpy as np
import pytest
import torch

from oracle import kv_fp8


def test_decode_known_codes():
    want = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x0F: 1.875 * 2.0 ** -6, 0x38: 1.0, 0x3C: 1.5,
            0x40: 2.0, 0x77: 1.875 * 2 ** 7, 0x78: 256.0, 0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0}
    for code, val in want.items():
        assert kv_fp8.e4m3_decode(np.uint8(code)) == val, hex(code)
    assert np.isnan(kv_fp8.e4m3_decode(np.uint8(0x7F))) and np.isnan(kv_fp8.e4m3_decode(np.uint8(0xFF)))
    z = kv_fp8.e4m3_decode(np.uint8(0x80))
    assert z == 0.0 and np.signbit(z)


def test_decode_all_codes_against_library_cast():
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = kv_fp8.e4m3_decode(codes)
    finite = ~np.isnan(lib)
    assert finite.sum() == 254 and np.array_equal(np.isnan(ours), ~finite)
    assert np.array_equal(ours[finite], lib[finite])
    # strictly increasing over the positive codes: the table has no duplicates and no gaps out of order
    assert np.all(np.diff(ours[:0x7F]) > 0)


def _nearest_by_brute_force(y):
    """The definition itself: the finite code whose value is nearest to y; of two equally near the one with the even
    code; beyond +-448 the largest code."""
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    vals = kv_fp8.e4m3_decode(codes)
    out = np.empty(len(y), np.uint8)
    for i, v in enumerate(y):
        side = codes[(codes >= 0x80) == bool(np.signbit(v))]
        sv = kv_fp8.e4m3_decode(side)
        d = np.abs(sv - v)
        best = np.flatnonzero(d == d.min())
        pick = [c for c in side[best] if c % 2 == 0] if len(best) > 1 else list(side[best])
        out[i] = pick[0]
    return out


def test_encode_is_nearest_with_ties_to_even_by_brute_force():
    g = np.random.default_rng(0)
    pos = kv_fp8.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    mid = (pos[:-1] + pos[1:]) / 2                                   # every tie point
    near = np.concatenate([mid * (1 + 2.0 ** -20), mid * (1 - 2.0 ** -20)])
    rnd = np.concatenate([g.uniform(-460, 460, 4000), g.standard_normal(4000), g.standard_normal(2000) * 2.0 ** -7,
                          g.uniform(-2.0 ** -8, 2.0 ** -8, 1000)])
    y = np.concatenate([pos, -pos, mid, -mid, near, -near, rnd, [448.0, 449.0, 463.9, 464.0, 1e9, -1e9, 0.0, -0.0]])
    assert np.array_equal(kv_fp8.e4m3_encode(y), _nearest_by_brute_force(y))


def test_encode_round_trips_every_code():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    assert np.array_equal(kv_fp8.e4m3_encode(kv_fp8.e4m3_decode(codes)), codes)


def test_encode_against_library_cast_in_range():
    g = np.random.default_rng(1)
    y = np.concatenate([g.uniform(-448, 448, 20000), g.standard_normal(20000) * 3, g.standard_normal(5000) * 2.0 ** -6])
    y = y.astype(np.float32)                                          # the library rounds from float32
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(kv_fp8.e4m3_encode(y), lib)


def test_block_exponent_is_the_smallest_that_fits():
    cases = {448.0: 0, 448.5: 1, 224.0: -1, 224.5: 0, 1.0: -8, 0.875: -9, 0.876: -8, 3.5: -7, 3.51: -6, 2.0 ** 20: 12}
    for amax, e in cases.items():
        assert kv_fp8.block_exponent(amax) == e, amax
    assert kv_fp8.block_exponent(0.0) == 0
    g = np.random.default_rng(2)
    for a in np.abs(g.standard_normal(2000)) * np.exp2(g.integers(-20, 20, 2000)):
        e = kv_fp8.block_exponent(a)
        assert a <= 448 * 2.0 ** e and a > 448 * 2.0 ** (e - 1)
    assert kv_fp8.block_exponent(1e-45) == -110 and kv_fp8.block_exponent(3e38) == 120


def test_quantize_blocks_and_error_bound():
    g = np.random.default_rng(3)
    H, n, D = 2, 150, 64                                              # two full blocks and a ragged one
    x = (g.standard_normal((H, n, D)) * np.exp2(g.integers(-3, 4, (H, n, 1)))).astype(np.float32)
    x[1, 64:128] = 0.0                                                # an all-zero block
    codes, exps = kv_fp8.quantize(x)
    assert codes.shape == x.shape and exps.shape == (H, 3) and exps[1, 1] == 0 and not codes[1, 64:128].any()
    for h in range(H):
        for b in range(3):
            blk = x[h, b * 64:(b + 1) * 64]
            if np.abs(blk).max() > 0:
                assert exps[h, b] == math.ceil(math.log2(np.abs(blk).max() / 448.0))   # the definition, in floating point
    back = kv_fp8.dequantize(codes, exps)
    scale = np.repeat(np.exp2(exps.astype(np.float64)), 64, axis=1)[:, :n, None]
    # half a code spacing: 2^-4 relative for normal codes, 2^-10 * scale absolute below the smallest normal
    assert np.all(np.abs(back - x) <= np.maximum(np.abs(x) * 2.0 ** -4, scale * 2.0 ** -10) * (1 + 1e-12))
    assert np.array_equal(kv_fp8.round_trip(x), back)
    # the largest element of a block uses the upper half of the code range
    top = np.abs(kv_fp8.e4m3_decode(codes)).reshape(H, -1)
    assert top[0].max() > 224


def test_append_requantises_only_from_the_open_block_on():
    g = np.random.default_rng(4)
    x = g.standard_normal((2, 200, 64)).astype(np.float32)
    x[:, 100:] *= 8.0                                      # later tokens raise the scale of the open block
    a = kv_fp8.round_trip(x[:, :70])
    b = kv_fp8.append(a, x[:, 70:150])
    assert b.shape == (2, 150, 64)
    assert np.array_equal(b[:, :64], a[:, :64])            # the full block before the open one is untouched
    # tokens appended on a block border are quantised as a slot of their own
    c = kv_fp8.append(kv_fp8.round_trip(x[:, :128]), x[:, 128:200])
    assert np.array_equal(c[:, 128:], kv_fp8.round_trip(x[:, 128:200])) and np.array_equal(c[:, :128], kv_fp8.round_trip(x[:, :128]))
    # the open block: same result as quantising [what was read back ; new tokens] in one go, and never further from the
    # source than one coarser rounding of the read-back values
    again = kv_fp8.round_trip(np.concatenate([a[:, 64:70], x[:, 70:128]], axis=1))
    assert np.array_equal(b[:, 64:128], again)
    # appending nothing-changing data is idempotent: values that are already codes at the block's scale stay put
    d = kv_fp8.append(a[:, :64], a[:, 64:70])
    assert np.array_equal(d, a)
