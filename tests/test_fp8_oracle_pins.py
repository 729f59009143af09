"""Pins for oracle/fp8_oracle.py (CPU only): the E4M3 format against its definition and published
constants, the encoder against a library conversion and a brute-force nearest search, and the
dynamic quantisation against invariants and an exactly representable case."""
import numpy as np
import torch

from oracle import fp8_oracle as F
from oracle import prefill_oracle as O


def test_decode_table_matches_the_format_definition():
    t = F.e4m3_decode(np.arange(256, dtype=np.uint8))
    # constants of the OCP 8-bit float specification for E4M3
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0               # largest finite
    assert t[0x08] == 2.0 ** -6                                  # smallest normal
    assert t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9     # smallest / largest subnormal
    assert t[0x38] == 1.0 and t[0x40] == 2.0 and t[0x3C] == 1.5
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.sum(np.isnan(t)) == 2     # no infinities
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and np.signbit(t[0x80])
    assert np.all(np.diff(t[:0x7F]) > 0)                         # codes order like magnitudes
    assert np.array_equal(t[0x80:0xFF], -t[:0x7F])
    # every value is (8 + m) * 2^(e - 10): 4 significant bits
    m, e = np.frexp(t[1:0x7F])
    assert np.all((m * 16) == np.round(m * 16))
    # against the library's decoder
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    assert np.array_equal(np.nan_to_num(lib, nan=12345.0), np.nan_to_num(t, nan=12345.0).astype(np.float32))


def test_encode_is_round_to_nearest_even():
    rng = np.random.default_rng(8)
    x = (rng.standard_normal(200000) * np.exp2(rng.integers(-12, 9, 200000))).astype(np.float32)
    x = x[np.abs(x) <= 464.0]
    got = F.e4m3_encode(x)
    # library conversion (same format, same rounding)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, lib)
    # brute force: nearest of the 127 non-negative values, ties to the even code
    vals = F.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    s = x[:3000].astype(np.float64)
    d = np.abs(np.abs(s)[:, None] - vals[None, :])
    best = np.min(d, axis=1)
    for i in range(len(s)):
        c = [j for j in range(0x7F) if d[i, j] == best[i]]
        pick = c[0] if len(c) == 1 else [j for j in c if j % 2 == 0][0]
        assert (got[i] & 0x7F) == pick and bool(got[i] & 0x80) == bool(np.signbit(s[i]))
    # all codes survive a round trip; every midpoint goes to its even neighbour
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    assert np.array_equal(F.e4m3_encode(F.e4m3_decode(codes).astype(np.float32)), codes)
    mid = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)
    enc = F.e4m3_encode(mid)
    assert np.all(enc % 2 == 0) and np.all(np.abs(enc.astype(int) - np.arange(0x7E)) <= 1)
    # the edge: 464 is the tie above the largest value, beyond it there is nothing to round to
    assert F.e4m3_encode(np.float32(464.0)) == 0x7E and F.e4m3_encode(np.float32(464.1)) == 0x7F
    assert F.e4m3_encode(np.float32(2.0 ** -10)) == 0x00 and F.e4m3_encode(np.float32(1.5 * 2.0 ** -10)) == 0x01


def test_quantize_rows_invariants():
    rng = np.random.default_rng(9)
    x = O.round_bf16(rng.standard_normal((64, 512)) * np.exp2(rng.integers(-6, 6, (64, 1))))
    x[5] = 0.0
    q, s = F.quantize_rows(x)
    assert q.dtype == np.uint8 and s.dtype == np.float32
    amax = np.max(np.abs(x), axis=1)
    # the largest element of a row takes the largest code; the scale is amax / 448 to one rounding
    j = np.argmax(np.abs(x), axis=1)
    rows = np.arange(64)
    assert np.all((q[rows, j] & 0x7F)[amax > 0] == 0x7E)
    assert np.all(np.abs(s.astype(np.float64)[amax > 0] * 448.0 / amax[amax > 0] - 1.0) <= 2.0 ** -23)
    assert np.all(q[5] == 0) and s[5] == 1.0
    # powers of two commute with everything: same codes, scaled scale
    q2, s2 = F.quantize_rows(x * 8.0)
    assert np.array_equal(q2, q) and np.array_equal(s2[amax > 0], s[amax > 0] * 8.0)
    # the stored values are within half a step (2^-4 relative, or half the subnormal step) of the inputs
    back = F.e4m3_decode(q) * s.astype(np.float64)[:, None]
    tol = np.maximum(np.abs(x) * 2.0 ** -4, (2.0 ** -10) * s.astype(np.float64)[:, None] * 1.0001)
    assert np.all(np.abs(back - x) <= tol * 1.0001)


def test_dynamic_linear_exact_case_and_error_bound():
    rng = np.random.default_rng(10)
    # values that are E4M3 numbers once their row is scaled to 448: the product must be exact
    grid = F.e4m3_decode(np.arange(0x30, 0x7F, dtype=np.uint8))
    x = rng.choice(grid, (16, 128)) * rng.choice([-1.0, 1.0], (16, 128))
    w = rng.choice(grid, (24, 128)) * rng.choice([-1.0, 1.0], (24, 128))
    x[:, 0] = 448.0
    w[:, 0] = -448.0
    x *= np.exp2(rng.integers(-8, 3, (16, 1)))
    w *= np.exp2(rng.integers(-8, 3, (24, 1)))
    assert np.array_equal(F.dynamic_linear(x, w), x @ w.T)
    # general inputs: every operand within 2^-4 relative => the product within a stated bound
    x = O.round_bf16(rng.standard_normal((32, 1024)))
    w = O.round_bf16(rng.standard_normal((48, 1024)) * 0.02)
    y, ref = F.dynamic_linear(x, w), x @ w.T
    bound = (2 * 2.0 ** -4 + 2.0 ** -8) * (np.abs(x) @ np.abs(w).T) + 1e-6
    assert np.all(np.abs(y - ref) <= bound)
    assert np.max(np.abs(y - ref)) / np.max(np.abs(ref)) < 0.06
    # an independent evaluation with the library's conversion
    def lib_q(a):
        a32 = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
        amax = a32.abs().amax(dim=1, keepdim=True)
        q8 = (a32 * (torch.tensor(448.0) / amax)).to(torch.float8_e4m3fn)
        return q8.to(torch.float64).numpy(), (amax / 448.0).to(torch.float64).numpy()
    (qx, sx), (qw, sw) = lib_q(x), lib_q(w)
    assert np.array_equal(y, (qx @ qw.T) * sx * sw.T)


def test_prefill_with_quantised_linears_differs_little_and_only_in_the_blocks():
    """The `linear` hook of the oracle: zero layers -> identical logits (the LM head is never quantised);
    with layers the logits move by a few percent of their range, not more."""
    import helpers as H
    from paper_2505_07203_amd import inputs as I
    cfg = I.TINY.replace(n_layers=0)
    tokens = I.make_tokens(cfg, 5, 40)
    z0, _ = H.oracle_prefill(cfg, 11, tokens)
    embed, fnorm, lm = H.oracle_globals(cfg, 11)
    z1, _ = O.prefill(tokens, embed, [], fnorm, lm, cfg, linear=F.dynamic_linear)
    assert np.array_equal(z0, z1)
    cfg = I.TINY
    za, _ = H.oracle_prefill(cfg, 11, tokens)
    embed, fnorm, lm = H.oracle_globals(cfg, 11)
    zb, _ = O.prefill(tokens, embed, H.oracle_layers(cfg, 11), fnorm, lm, cfg, linear=F.dynamic_linear)
    rel = np.max(np.abs(za - zb)) / np.max(np.abs(za))
    assert 1e-4 < rel < 0.2, rel
