"""Reference for the 8-bit K/V slot format.  TEST INFRASTRUCTURE ONLY: only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import this package; it shares nothing with the HIP library.

The paper stores the chunks' complete tensors and leaves other cache organisations to future work (Sec. 7, fine-grained
cache organisation); this format is the library's smaller variant of a slot, defined here so that both sides can be
checked bit for bit:

  * element code: E4M3 of the OCP 8-bit floating point specification -- 1 sign bit, 4 exponent bits (bias 7),
    3 mantissa bits, no infinities, S.1111.111 is NaN, largest finite magnitude 448, subnormals m/8 * 2^-6;
    conversion rounds to nearest, ties to the even code, and saturates at +-448;
  * one power-of-two scale 2^e per (kv head, block of 64 tokens), separately for K and for V:
    e is the smallest integer with  max|x| <= 448 * 2^e  over the block's stored tokens (0 for an all-zero block),
    kept inside [-110, 127] (so that every value read back is a normal bf16 number); the stored code of x is
    E4M3(x * 2^-e) and the value read back is code * 2^e.

  * appending tokens to a slot that holds n: everything from the block that contains token n on is quantised afresh
    from the values the slot currently reads back plus the new tokens (full blocks before it stay as they are).

Everything is computed in float64 on values that are exactly representable, so no step rounds except the one the
format defines.  parity unpinned by the paper (it prints no such format); pinned by tests/test_oracle_kv_fp8.py against
the format's definition by brute force and against a library conversion routine.
"""
from __future__ import annotations

import math

import numpy as np

BLOCK = 64          # tokens per scale
E4M3_MAX = 448.0


def e4m3_decode(code) -> np.ndarray:
    """Value of each 8-bit code (float64; NaN for the two NaN codes)."""
    c = np.asarray(code, np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    ex = (c >> 3) & 0xF
    man = c & 0x7
    normal = (1.0 + man / 8.0) * np.exp2(ex.astype(np.float64) - 7.0)
    sub = (man / 8.0) * 2.0 ** -6
    val = np.where(ex == 0, sub, normal)
    val = np.where((ex == 15) & (man == 7), np.nan, val)
    return sign * val


def e4m3_encode(y) -> np.ndarray:
    """Nearest code of each value (ties to the even code), saturating at +-448.  -0.0 keeps its sign."""
    y = np.asarray(y, np.float64)
    a = np.minimum(np.abs(y), E4M3_MAX)
    # spacing of the codes around a: 2^(E-3) in the binade [2^E, 2^(E+1)), E >= -6; 2^-9 below 2^-6
    _, ex = np.frexp(np.where(a > 0, a, 1.0))          # a = m * 2^ex, m in [0.5, 1)  ->  E = ex - 1
    E = np.maximum(ex - 1, -6)
    quantum = np.exp2(E.astype(np.float64) - 3.0)
    q = np.rint(a / quantum)                            # half to even; exact: a / quantum is a small binary fraction
    # q in [0, 16]; q == 16 is the first value of the next binade
    up = q == 16
    E = np.where(up, E + 1, E)
    q = np.where(up, 8.0, q)
    normal = q >= 8
    field = np.where(normal, E + 7, 0).astype(np.int64)
    man = np.where(normal, q - 8, q).astype(np.int64)
    code = (field << 3) | man
    code = np.where(np.signbit(y), code | 0x80, code)
    return code.astype(np.uint8)


def block_exponent(amax: float) -> int:
    """Smallest e with amax <= 448 * 2^e (0 for amax == 0), kept inside [-110, 127]."""
    if amax == 0:
        return 0
    m, k = math.frexp(float(amax))                      # amax = m * 2^k, m in [0.5, 1);  448 = 0.875 * 2^9
    e = k - 9 if m <= 0.875 else k - 8
    return max(-110, min(127, e))


def quantize(x):
    """x [heads, n_tokens, D] (values of the storage dtype) -> (codes uint8 of the same shape,
    exponents int32 [heads, ceil(n_tokens / 64)])."""
    x = np.asarray(x, np.float64)
    H, n, D = x.shape
    nb = (n + BLOCK - 1) // BLOCK
    codes = np.zeros((H, n, D), np.uint8)
    exps = np.zeros((H, nb), np.int32)
    for h in range(H):
        for b in range(nb):
            blk = x[h, b * BLOCK:(b + 1) * BLOCK]
            e = block_exponent(float(np.abs(blk).max()))
            exps[h, b] = e
            codes[h, b * BLOCK:(b + 1) * BLOCK] = e4m3_encode(blk * 2.0 ** -e)
    return codes, exps


def dequantize(codes, exps) -> np.ndarray:
    """The values a slot holds: code * 2^e (float32, exact)."""
    codes = np.asarray(codes, np.uint8)
    H, n, D = codes.shape
    scale = np.repeat(np.exp2(np.asarray(exps, np.float64)), BLOCK, axis=1)[:, :n]
    return (e4m3_decode(codes) * scale[:, :, None]).astype(np.float32)


def round_trip(x) -> np.ndarray:
    """What a slot returns for x: quantize, then dequantize."""
    return dequantize(*quantize(x))


def append(stored, new) -> np.ndarray:
    """stored [heads, n, D]: what the slot reads back now; new [heads, m, D]: tokens of the storage dtype to append.
    Returns what the slot reads back afterwards ([heads, n + m, D])."""
    stored = np.asarray(stored, np.float32)
    new = np.asarray(new, np.float32)
    n = stored.shape[1]
    first = (n // BLOCK) * BLOCK
    tail = np.concatenate([stored[:, first:], new], axis=1)
    return np.concatenate([stored[:, :first], round_trip(tail)], axis=1)
