"""CPU oracle for the FP8-dynamic variant of the decoder's linear layers.  TEST INFRASTRUCTURE ONLY.

The paper evaluates FP8-dynamic checkpoints on its larger GPUs (Section 7.1, hardware / model
table) without defining the scheme; the reading taken here is the public convention those
checkpoints follow:

  * number format: OCP 8-bit float E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits;
    exponent field 0 = subnormals m * 2^-9; no infinities; S.1111.111 is NaN; largest finite
    value 448);
  * weights: one float32 scale per output channel (row of W [out, in]), fixed at load time;
  * activations: one float32 scale per token (row), computed from that row when it is used;
  * a row x with amax = max|x_k| is stored as codes q_k = e4m3(x_k * (448 / amax)) and the scale
    s = amax / 448 (amax == 0: codes 0, scale 1); both divisions and the product are single
    float32 operations, the conversion rounds to nearest with ties to even (a magnitude above 464,
    which dynamic scaling never produces, becomes NaN);
  * y[m, n] = (sum_k q_x[m, k] * q_w[n, k]) * s_x[m] * s_w[n]  (+ bias), the sum exact here
    (float64 over at most 2^16 products of 7-bit-significand values).

Only the decoder blocks' linear layers (Q/K/V, O, gate/up, down) are quantised; embedding,
norms, rotary embedding, attention and the LM head are untouched.  Everything here is plain
numpy; nothing is shared with the HIP library.  Pins: tests/test_fp8_oracle_pins.py (the decode
table against the format's definition and its published constants, the encoder against a
library conversion and a brute-force nearest search, ties, subnormals, scaling invariants).
"""
from __future__ import annotations

import numpy as np

__all__ = ["E4M3_MAX", "e4m3_decode", "e4m3_encode", "quantize_rows", "dynamic_linear"]

E4M3_MAX = 448.0


def _decode_table() -> np.ndarray:
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            t[code] = np.nan
        elif e == 0:
            t[code] = sign * m * 2.0 ** -9
        else:
            t[code] = sign * (8 + m) * 2.0 ** (e - 10)
    return t


_TABLE = _decode_table()
_POS = _TABLE[:0x7F]                                   # codes 0x00 .. 0x7E: 0, 2^-9, ..., 448 (increasing)
_MID = (_POS[:-1] + _POS[1:]) / 2.0                    # midpoints between neighbours (exact in float64)
_TOP = (448.0 + 480.0) / 2.0                           # midpoint to the value the NaN code displaces


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """uint8 codes -> float64 values (NaN for 0x7F / 0xFF)."""
    return _TABLE[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """float32 values -> uint8 E4M3 codes: nearest representable value, ties to the even code;
    a magnitude above 464 (the midpoint to the first value the format lacks) gives NaN (0x7F);
    exactly 464 is a tie and goes to the even neighbour, 448."""
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    a = np.abs(x)
    idx = np.searchsorted(_MID, a, side="left")        # first code whose upper midpoint is >= a
    # a == _MID[idx]: tie between codes idx and idx + 1 -> the even one
    tie = (idx < len(_MID)) & (a == _MID[np.minimum(idx, len(_MID) - 1)])
    idx = np.where(tie & (idx % 2 == 1), idx + 1, idx)
    code = idx.astype(np.uint8)
    code = np.where(a > _TOP, np.uint8(0x7F), code)
    code = np.where(np.isnan(a), np.uint8(0x7F), code)
    return (code | np.where(np.signbit(x), np.uint8(0x80), np.uint8(0))).astype(np.uint8)


def quantize_rows(x: np.ndarray):
    """Rows of x -> (codes uint8 [M, K], scales float32 [M]).  x is taken as its nearest float32
    (bf16 activations and weights are float32 values already); all arithmetic before the
    conversion is float32, one rounding per operation."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    amax = np.max(np.abs(x32), axis=1)
    safe = np.where(amax > 0, amax, np.float32(1)).astype(np.float32)
    inv = (np.float32(E4M3_MAX) / safe).astype(np.float32)
    scale = np.where(amax > 0, (safe / np.float32(E4M3_MAX)).astype(np.float32), np.float32(1)).astype(np.float32)
    codes = e4m3_encode((x32 * inv[:, None]).astype(np.float32))
    return codes, scale


def dynamic_linear(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """y = x W^T with both operands stored as E4M3: per-token scales for x [M, K], per-output-
    channel scales for W [N, K]; float64 result."""
    qx, sx = quantize_rows(x)
    qw, sw = quantize_rows(w)
    acc = e4m3_decode(qx) @ e4m3_decode(qw).T
    return acc * sx.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :]
