"""Parity at the sizes and launch configurations the benchmark times (Llama-3-8B shape, 32768
tokens, MLP chunk 4096): outputs the oracle can compute one by one, and properties that hold
at any size.

  * attention over the whole 32768-token sequence in one launch: sampled query rows (first
    and last rows of tiles, rows next to the diagonal, the last row) against the oracle's
    definition evaluated for exactly those rows;
  * the three fused GEMMs at their benchmark shapes: whole sampled rows (every column tile)
    and whole sampled columns (every row tile) against float64 matrix products;
  * the whole path: bit-identical logits across MLP chunk sizes and across repeated runs;
  * the same for the other two large workloads' launch shapes: attention over 131072 tokens (sampled rows in
    the first, middle and last query tiles), attention with five query heads per KV head over 16384 tokens,
    the Qwen-32B-shaped GEMMs, and a two-layer whole-path run at 131072 tokens with every layer computed in full;
  * attention inputs with one key far above all earlier ones inside a key block (the case in which the fast
    kernel's fixed reference exponent gives up and the tile is recomputed with a running maximum).
"""
import numpy as np
import pytest
import torch

from paper_2505_07203_amd import binding as B
from paper_2505_07203_amd import inputs as I
from oracle import prefill_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def bf16_dev(x32: np.ndarray):
    """float32 array -> (device bf16 tensor, the same values as float64)"""
    bits = I.f32_to_bf16_bits(x32)
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return t, I.stored_to_f64(bits)


def host64(t) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def q_operand(qs32: np.ndarray, prescaled: bool):
    """-> (device bf16 queries as the attention entry point takes them, the queries the definition sees, float64).
    prescaled: the stored values are bf16(q * log2(e) / sqrt(hd)), the form the full path hands to attention; the
    definition then sees those stored values divided by the scale."""
    if not prescaled:
        return bf16_dev(qs32)
    c = np.float32(B.attention_q_scale(qs32.shape[-1]))
    t, stored = bf16_dev(qs32 * c)
    return t, stored / np.float64(c)


# ------------------------------------------------------------------ attention, 32768 tokens

@pytest.mark.parametrize("prescaled", [False, True], ids=["q", "q_prescaled"])
def test_attention_32k_sampled_rows(prescaled):
    N, Hq, Hkv, hd = 32768, 32, 8, 128
    rng = np.random.default_rng(32768)
    q, q64 = q_operand(rng.standard_normal((N, Hq, hd), dtype=np.float32), prescaled)
    k, k64 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    v, v64 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    rows = np.array([0, 1, 31, 32, 63, 64, 65, 127, 255, 256, 257, 319, 4095, 4096, 12345, 16383, 16384,
                     20000, 32511, 32512, 32575, 32703, 32766, 32767])
    ref = O.causal_gqa_attention(q64, k64, v64, query_rows=rows)
    del q64
    got = host64(B.po_op_attention(q, k, v, q_prescaled=prescaled)[torch.from_numpy(rows).cuda()])
    err = np.max(np.abs(got - ref), axis=(1, 2)) / np.max(np.abs(ref))
    print("attention N=32768, per sampled row:", " ".join(f"{r}:{e:.1e}" for r, e in zip(rows, err)))
    assert np.max(err) <= 1.5e-2


def test_attention_float32_32k_sampled_rows():
    """The float32 path's attention (the float32 matrix instruction) at the benchmark's length and head layout: it
    stands in for the float64 definition at whole configurations, so it is held to float32 rounding here."""
    N, Hq, Hkv, hd = 32768, 32, 8, 128
    rng = np.random.default_rng(32769)
    q, k, v = (rng.standard_normal((N, h, hd), dtype=np.float32) for h in (Hq, Hkv, Hkv))
    rows = np.array([0, 1, 31, 32, 33, 63, 64, 127, 128, 129, 255, 4095, 4096, 12345, 16383, 16384, 20000, 32639, 32640,
                     32671, 32672, 32735, 32766, 32767])
    ref = O.causal_gqa_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), query_rows=rows)
    dq = torch.from_numpy(q).cuda()
    got = B.po_op_attention(dq, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda())
    got = got[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    err = np.max(np.abs(got - ref), axis=(1, 2)) / np.max(np.abs(ref))
    print("float32 attention N=32768, per sampled row:", " ".join(f"{r}:{e:.1e}" for r, e in zip(rows, err)))
    assert np.max(err) <= 2e-5


@pytest.mark.parametrize("prescaled", [False, True], ids=["q", "q_prescaled"])
def test_attention_large_scores_renormalise(prescaled):
    """Scores far above the first key block's maximum: the running sums pass the
    renormalisation threshold many times (with prescaled queries, which use no reference exponent, the rows whose
    sums leave the float range are recomputed with a running maximum instead)."""
    N, Hq, Hkv, hd = 2048, 8, 2, 128
    rng = np.random.default_rng(7)
    qs = rng.standard_normal((N, Hq, hd), dtype=np.float32)
    ks = rng.standard_normal((N, Hkv, hd), dtype=np.float32)
    # growing key norm: later keys score higher and higher than the early ones
    ks *= (1.0 + 7.0 * np.arange(N, dtype=np.float32) / N)[:, None, None]
    qs *= 3.0
    q, q64 = q_operand(qs, prescaled)
    k, k64 = bf16_dev(ks)
    v, v64 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    ref = O.causal_gqa_attention(q64, k64, v64)
    got = host64(B.po_op_attention(q, k, v, q_prescaled=prescaled))
    assert np.all(np.isfinite(got))
    err = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
    print(f"attention with large scores: {err:.3e}")
    assert err <= 1.5e-2


@pytest.mark.parametrize("prescaled", [False, True], ids=["q", "q_prescaled"])
@pytest.mark.parametrize("nats", [70.0, 150.0, 400.0])
def test_attention_outlier_key_mid_block(nats, prescaled):
    """One key, in the middle of a 32-key block, scores `nats` above everything before it for every query.
    70 nats (101 in log2 units) is inside what one block's exponentials hold: the row sums are renormalised.
    150 and 400 nats overflow the exponential against the reference taken from the first block: those query
    tiles must be recomputed with a running maximum.  The definition (oracle) gives, for rows at or after the
    outlier, almost exactly that key's value; the output must be finite and match, also when it overwrites Q."""
    N, Hq, Hkv, hd = 1024, 8, 2, 128
    pos = 19 * 32 + 13
    rng = np.random.default_rng(int(nats))
    qs = rng.standard_normal((N, Hq, hd), dtype=np.float32)
    ks = rng.standard_normal((N, Hkv, hd), dtype=np.float32)
    qs[:, :, 0] = 8.0
    ks[pos, :, 0] = np.float32(nats) * np.sqrt(np.float32(hd)) / 8.0
    q, q64 = q_operand(qs, prescaled)
    k, k64 = bf16_dev(ks)
    v, v64 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    ref = O.causal_gqa_attention(q64, k64, v64)
    # the oracle itself: behind the outlier the softmax is that key alone
    assert np.max(np.abs(ref[pos:] - v64[pos][None].repeat(Hq // Hkv, axis=1))) < 1e-6
    got = host64(B.po_op_attention(q, k, v, q_prescaled=prescaled))
    assert np.all(np.isfinite(got))
    err = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
    print(f"attention with a key {nats} nats above its predecessors: {err:.3e}")
    assert err <= 1.5e-2
    dq = q.clone()
    B.po_op_attention(dq, k, v, out=dq, q_prescaled=prescaled)
    assert np.array_equal(host64(dq), got)
    # and the next call on ordinary inputs is unaffected (the give-up words were left clean)
    k2, k264 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    ref2 = O.causal_gqa_attention(q64, k264, v64)
    got2 = host64(B.po_op_attention(q, k2, v, q_prescaled=prescaled))
    assert np.max(np.abs(got2 - ref2)) / np.max(np.abs(ref2)) <= 1.5e-2


@pytest.mark.parametrize("prescaled", [False, True], ids=["q", "q_prescaled"])
@pytest.mark.parametrize("nats", [-45.0, -150.0])
def test_attention_all_scores_far_below_zero(nats, prescaled):
    """Every score of every row sits `nats` below zero (a common component of all keys against a common component
    of all queries).  Softmax does not care; an implementation that exponentiates without a reference would flush
    the probabilities to zero.  With prescaled queries the kernel's row sums fall below its floor and the tiles are
    recomputed with a running maximum."""
    N, Hq, Hkv, hd = 700, 8, 2, 128
    rng = np.random.default_rng(int(-nats))
    qs = rng.standard_normal((N, Hq, hd), dtype=np.float32)
    ks = rng.standard_normal((N, Hkv, hd), dtype=np.float32)
    qs[:, :, 0] = 8.0
    ks[:, :, 0] = np.float32(nats) * np.sqrt(np.float32(hd)) / 8.0
    q, q64 = q_operand(qs, prescaled)
    k, k64 = bf16_dev(ks)
    v, v64 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    ref = O.causal_gqa_attention(q64, k64, v64)
    got = host64(B.po_op_attention(q, k, v, q_prescaled=prescaled))
    assert np.all(np.isfinite(got))
    err = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
    print(f"attention with all scores {nats} nats: {err:.3e}")
    assert err <= 1.5e-2


@pytest.mark.parametrize("prescaled", [False, True], ids=["q", "q_prescaled"])
def test_attention_128k_sampled_rows(prescaled):
    """The 131072-token workload's attention launch (32 query heads, 8 KV heads): rows of the first, middle
    and last query tiles against the definition evaluated for exactly those rows."""
    N, Hq, Hkv, hd = 131072, 32, 8, 128
    rng = np.random.default_rng(131072)
    q, q64 = q_operand(rng.standard_normal((N, Hq, hd), dtype=np.float32), prescaled)
    k, k64 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    v, v64 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    rows = np.array([0, 1, 63, 64, 255, 256, 257, 511, 32767, 32768, 65535, 65536, 65537, 65599, 65791, 70001,
                     98304, 130815, 130816, 130879, 130880, 131007, 131070, 131071])
    ref = O.causal_gqa_attention(q64, k64, v64, query_rows=rows)
    del q64
    got = host64(B.po_op_attention(q, k, v, q_prescaled=prescaled)[torch.from_numpy(rows).cuda()])
    err = np.max(np.abs(got - ref), axis=(1, 2)) / np.max(np.abs(ref))
    print("attention N=131072, per sampled row:", " ".join(f"{r}:{e:.1e}" for r, e in zip(rows, err)))
    assert np.max(err) <= 1.5e-2


@pytest.mark.parametrize("prescaled", [False, True], ids=["q", "q_prescaled"])
def test_attention_qwen_heads_16k_sampled_rows(prescaled):
    """Five query heads per KV head (40 and 8) over 16384 tokens: the Qwen-32B-shaped workload's launch."""
    N, Hq, Hkv, hd = 16384, 40, 8, 128
    rng = np.random.default_rng(16384)
    q, q64 = q_operand(rng.standard_normal((N, Hq, hd), dtype=np.float32), prescaled)
    k, k64 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    v, v64 = bf16_dev(rng.standard_normal((N, Hkv, hd), dtype=np.float32))
    rows = np.array([0, 31, 32, 255, 256, 1000, 4095, 4096, 8191, 8192, 12345, 16127, 16128, 16191, 16382, 16383])
    ref = O.causal_gqa_attention(q64, k64, v64, query_rows=rows)
    got = host64(B.po_op_attention(q, k, v, q_prescaled=prescaled)[torch.from_numpy(rows).cuda()])
    # every query head must have read ITS KV head: compare head by head
    err = np.max(np.abs(got - ref), axis=(0, 2)) / np.max(np.abs(ref))
    print("attention N=16384, 40/8 heads, per query head:", " ".join(f"{e:.1e}" for e in err))
    assert np.max(err) <= 1.5e-2


# ------------------------------------------------------------------ GEMMs at benchmark shapes

ROWS = np.array([0, 1, 255, 256, 257, 2047, 4094, 4095])


def _check_rows_cols(got, ref_rows, ref_cols, rows, cols, tol):
    scale = max(np.max(np.abs(ref_rows)), np.max(np.abs(ref_cols)))
    e_r = np.max(np.abs(got[rows] - ref_rows)) / scale
    e_c = np.max(np.abs(got[:, cols] - ref_cols)) / scale
    assert e_r <= tol and e_c <= tol, (e_r, e_c)
    return max(e_r, e_c)


@pytest.mark.parametrize("shape", [(4096, 4096, 4096), (4096, 4096, 14336), (4096, 5120, 5120), (4096, 5120, 27648),
                                   (3072, 5120, 27648)],
                         ids=lambda t: "x".join(map(str, t)))
def test_gemm_residual_benchmark_shapes(shape):
    """O-projection and MLP down projection with the residual added in place: Llama-3-8B shape (K = 4096,
    14336) and Qwen2.5-32B shape (N = 5120, K = 5120, 27648; 3072 rows is what the path launches there)."""
    for M, N, K in (shape,):
        rng = np.random.default_rng(K)
        a, a64 = bf16_dev(rng.standard_normal((M, K), dtype=np.float32))
        w, w64 = bf16_dev(rng.standard_normal((N, K), dtype=np.float32) * 0.02)
        r, r64 = bf16_dev(rng.standard_normal((M, N), dtype=np.float32))
        cols = np.array([0, 63, 64, 255, 256, 2049, N - 64, N - 1])
        ROWS = np.array([0, 1, 255, 256, 257, 2047, M - 2, M - 1])
        ref_rows = a64[ROWS] @ w64.T + r64[ROWS]
        ref_cols = a64 @ w64[cols].T + r64[:, cols]
        B.po_op_linear(a, w, residual=r, out=r)
        e = _check_rows_cols(host64(r), ref_rows, ref_cols, ROWS, cols, 6e-3)
        print(f"residual GEMM {M}x{N}x{K}: {e:.2e}")


@pytest.mark.parametrize("shape", [(4096, 14336, 4096), (4096, 27648, 5120)], ids=lambda t: "x".join(map(str, t)))
def test_gemm_gate_up_silu_benchmark_shape(shape):
    """Gate/up projection with the SiLU-multiply: Llama-3-8B shape and Qwen2.5-32B shape (4096 x 55296 x 5120)."""
    M, F, K = shape
    rng = np.random.default_rng(F)
    a, a64 = bf16_dev(rng.standard_normal((M, K), dtype=np.float32))
    wg, g64 = bf16_dev(rng.standard_normal((F, K), dtype=np.float32) * 0.02)
    wu, u64 = bf16_dev(rng.standard_normal((F, K), dtype=np.float32) * 0.02)
    cols = np.array([0, 31, 32, 63, 64, 7000, F - 32, F - 1])

    def mlp_act(x, gw, uw):
        gate, up = x @ gw.T, x @ uw.T
        return gate / (1 + np.exp(-gate)) * up
    ref_rows = mlp_act(a64[ROWS], g64, u64)
    ref_cols = mlp_act(a64, g64[cols], u64[cols])
    got = host64(B.po_op_gate_up_silu(a, B.po_op_pack_gate_up(wg, wu)))
    e = _check_rows_cols(got, ref_rows, ref_cols, ROWS, cols, 6e-3)
    print(f"gate/up GEMM {M}x{2 * F}x{K}: {e:.2e}")


@pytest.mark.parametrize("shape", [(8192, 32, 8, 4096, 24576, 500000.0), (8192, 40, 8, 5120, 8192, 1000000.0)],
                         ids=["llama8b", "qwen32b"])
def test_gemm_qkv_rope_benchmark_shape(shape):
    """8192-row QKV projection with RoPE (Llama-3-8B shape at positions 24576 .. 32767; Qwen2.5-32B shape,
    8192 x 7168 x 5120, at positions 8192 .. 16383), V written transposed."""
    M, Hq, Hkv, K, pos0, theta = shape
    hd = 128
    rng = np.random.default_rng(M)
    a, a64 = bf16_dev(rng.standard_normal((M, K), dtype=np.float32))
    wq, q64 = bf16_dev(rng.standard_normal((Hq * hd, K), dtype=np.float32) * 0.02)
    wk, k64 = bf16_dev(rng.standard_normal((Hkv * hd, K), dtype=np.float32) * 0.02)
    wv, v64 = bf16_dev(rng.standard_normal((Hkv * hd, K), dtype=np.float32) * 0.02)
    rows = np.array([0, 1, 255, 256, 4095, 4096, 8190, 8191])
    pos = pos0 + rows
    ref_q = O.rope((a64[rows] @ q64.T).reshape(len(rows), Hq, hd), pos, theta)
    ref_k = O.rope((a64[rows] @ k64.T).reshape(len(rows), Hkv, hd), pos, theta)
    ref_v = a64[rows] @ v64.T
    cos, sin = B.po_op_rope_table(pos0 + M, hd, theta)
    wqkv, _ = B.po_op_pack_qkv(wq, wk, wv, Hq, Hkv, hd)
    c = B.attention_q_scale(hd)
    q, k, vt = B.po_op_qkv_rope(a, wqkv, None, cos, sin, Hq, Hkv, hd, pos0=pos0, q_scale=c)     # as the full path calls it
    ref_q = ref_q * c
    gq = host64(q).reshape(M, Hq, hd)[rows]
    gk = host64(k).reshape(M, Hkv, hd)[rows]
    gv = host64(vt)[:, pos].T if vt.shape[1] > M else host64(vt)[:, rows].T
    for name, g, r in (("q", gq, ref_q), ("k", gk, ref_k), ("v", gv, ref_v)):
        e = np.max(np.abs(g - r)) / np.max(np.abs(r))
        print(f"qkv+rope {name}: {e:.2e}")
        assert e <= 6e-3, (name, e)


def test_gemm_tile_heights_give_the_same_bits():
    """The bf16 GEMM picks 128-row or 256-row block tiles by how many tiles a launch has.  Every output is one fp32
    accumulator running over K in the same order in both forms, so the rows of a short launch (128-row tiles) must
    equal, bit for bit, the same rows inside a long launch (256-row tiles) -- what the chunk, prefix-cache and packing
    invariances of the path rest on (Section 4.2: chunking leaves the result unchanged).  All three fused epilogues,
    a ragged row count included."""
    rng = np.random.default_rng(77)
    big, small = 4096, 1100                                          # 16 x 16 tiles of 256 rows; 9 x 16 tiles of 128
    a, _ = bf16_dev(rng.standard_normal((big, 4096), dtype=np.float32))
    w, _ = bf16_dev(rng.standard_normal((4096, 4096), dtype=np.float32) * 0.02)
    r, _ = bf16_dev(rng.standard_normal((big, 4096), dtype=np.float32))
    full = B.po_op_linear(a, w, residual=r)
    part = B.po_op_linear(a[:small].contiguous(), w, residual=r[:small].contiguous())
    assert torch.equal(full[:small], part)
    # gate/up + SiLU-multiply: 256 rows x 112 column tiles take the 128-row form, 4096 rows the 256-row form
    wg, _ = bf16_dev(rng.standard_normal((14336, 4096), dtype=np.float32) * 0.02)
    wu, _ = bf16_dev(rng.standard_normal((14336, 4096), dtype=np.float32) * 0.02)
    wgu = B.po_op_pack_gate_up(wg, wu)
    full = B.po_op_gate_up_silu(a, wgu)
    part = B.po_op_gate_up_silu(a[:200].contiguous(), wgu)
    assert torch.equal(full[:200], part)
    # QKV + RoPE + transposed V: 1000 rows x 24 column tiles against 8192 rows
    Hq, Hkv, hd = 32, 8, 128
    a8, _ = bf16_dev(rng.standard_normal((8192, 4096), dtype=np.float32))
    wq, _ = bf16_dev(rng.standard_normal((Hq * hd, 4096), dtype=np.float32) * 0.02)
    wk, _ = bf16_dev(rng.standard_normal((Hkv * hd, 4096), dtype=np.float32) * 0.02)
    wv, _ = bf16_dev(rng.standard_normal((Hkv * hd, 4096), dtype=np.float32) * 0.02)
    cos, sin = B.po_op_rope_table(8192, hd, 500000.0)
    wqkv, _ = B.po_op_pack_qkv(wq, wk, wv, Hq, Hkv, hd)
    c = B.attention_q_scale(hd)
    q, k, vt = B.po_op_qkv_rope(a8, wqkv, None, cos, sin, Hq, Hkv, hd, pos0=0, q_scale=c)
    q2, k2, vt2 = B.po_op_qkv_rope(a8[:1000].contiguous(), wqkv, None, cos, sin, Hq, Hkv, hd, pos0=0, q_scale=c)
    assert torch.equal(q[:1000], q2) and torch.equal(k[:1000], k2) and torch.equal(vt[:, :1000], vt2[:, :1000])


# ------------------------------------------------------------------ whole path at 32768 tokens

def test_full_path_32k_bitwise_properties():
    """Two layers of the 8B shape on the benchmark's 32768 tokens: logits identical bit for bit for MLP
    chunks 4096 (the benchmark's), 8192 and 3000 (ragged last chunk), and across repeated runs."""
    w = I.WORKLOADS["llama8b_32k"]
    cfg = w["cfg"].replace(n_layers=2)
    tokens = I.make_tokens(cfg, w["tseed"], 32768, request=0)
    cand = I.label_ids(cfg)
    outs = []
    for chunk in (4096, 8192, 3000):
        ctx = B.Context(cfg, 32768, chunk)
        try:
            ctx.load_synthetic(w["wseed"], threads=16)
            z, lp = ctx.po_prefill(tokens, cand, want_logits=True)
            if chunk == 4096:
                z2, lp2 = ctx.po_prefill(tokens, cand, want_logits=True)
                assert np.array_equal(z, z2) and np.array_equal(lp, lp2)
            outs.append((z, lp))
        finally:
            ctx.po_destroy()
    assert np.all(np.isfinite(outs[0][0]))
    for z, lp in outs[1:]:
        assert np.array_equal(z, outs[0][0]) and np.array_equal(lp, outs[0][1])


def test_full_path_128k_bitwise_properties():
    """Two layers of the 8B shape on the 131072-token workload, BOTH computed in full (last-layer shortcut off,
    so the second layer's attention runs all 512 query tiles over the first layer's output): finite logits,
    identical bit for bit for MLP chunks 8192 (that workload's) and 4096, and with the shortcut on."""
    w = I.WORKLOADS["llama8b_128k"]
    cfg = w["cfg"].replace(n_layers=2)
    tokens = I.make_tokens(cfg, w["tseed"], 131072, request=0)
    cand = I.label_ids(cfg)
    outs = []
    for chunk, lazy in ((8192, False), (4096, False), (8192, True)):
        ctx = B.Context(cfg, 131072, chunk)
        try:
            ctx.load_synthetic(w["wseed"], threads=16)
            ctx.po_set_lazy_last_layer(lazy)
            outs.append(ctx.po_prefill(tokens, cand, want_logits=True))
        finally:
            ctx.po_destroy()
    assert np.all(np.isfinite(outs[0][0]))
    for z, lp in outs[1:]:
        assert np.array_equal(z, outs[0][0]) and np.array_equal(lp, outs[0][1])


# ------------------------------------------------------------------ FP8-dynamic GEMMs at benchmark shapes

def _fp8_operand(rng, rows, K, scale):
    """bf16 random matrix -> (device codes, device scales, decoded codes float64 [rows, K], scales float64)"""
    from oracle import fp8_oracle as F
    t, _ = bf16_dev(rng.standard_normal((rows, K), dtype=np.float32) * scale)
    q, s = B.po_op_quantize_rows(t)
    return q, s, F.e4m3_decode(q.cpu().numpy()), s.cpu().numpy().astype(np.float64)


def test_gemm_fp8_benchmark_shapes():
    """The FP8 MFMA GEMM at the shapes `bench.py --fp8` times (O-projection, down projection with the residual
    added in place, gate/up with the SiLU-multiply): whole sampled rows and columns against the exact sum of
    the same codes.  Tolerance: bf16 rounding of the result (2^-8) plus fp32 accumulation of K products."""
    for M, N, K, silu in ((4096, 4096, 4096, False), (4096, 4096, 14336, False), (4096, 2 * 14336, 4096, True)):
        rng = np.random.default_rng(N + K)
        qa, sa_d, aq, sa = _fp8_operand(rng, M, K, 1.0)
        if silu:
            Fd = N // 2
            qg, sg_d, gq, sg = _fp8_operand(rng, Fd, K, 0.02)
            qu, su_d, uq, su = _fp8_operand(rng, Fd, K, 0.02)
            def pack(g, u):
                return torch.stack((g.view(Fd // 32, 32, *g.shape[1:]), u.view(Fd // 32, 32, *u.shape[1:])),
                                   dim=1).reshape(2 * Fd, *g.shape[1:]).contiguous()
            got = host64(B.po_op_linear_fp8(qa, sa_d, pack(qg, qu), pack(sg_d, su_d), silu_mul=True))
            cols = np.array([0, 31, 32, 63, 64, 7000, 14304, 14335])

            def act(a_, sa_, gw, sgw, uw, suw):
                gate = (a_ @ gw.T) * sa_[:, None] * sgw[None, :]
                up = (a_ @ uw.T) * sa_[:, None] * suw[None, :]
                return gate / (1 + np.exp(-gate)) * up
            ref_rows = act(aq[ROWS], sa[ROWS], gq, sg, uq, su)
            ref_cols = act(aq, sa, gq[cols], sg[cols], uq[cols], su[cols])
            e = _check_rows_cols(got, ref_rows, ref_cols, ROWS, cols, 6e-3)
        else:
            qw, sw_d, wq, sw = _fp8_operand(rng, N, K, 0.02)
            r, r64 = bf16_dev(rng.standard_normal((M, N), dtype=np.float32))
            cols = np.array([0, 63, 64, 255, 256, 2049, 4032, 4095])
            ref_rows = (aq[ROWS] @ wq.T) * sa[ROWS, None] * sw[None, :] + r64[ROWS]
            ref_cols = (aq @ wq[cols].T) * sa[:, None] * sw[None, cols] + r64[:, cols]
            B.po_op_linear_fp8(qa, sa_d, qw, sw_d, residual=r, out=r)
            e = _check_rows_cols(host64(r), ref_rows, ref_cols, ROWS, cols, 6e-3)
        print(f"fp8 GEMM {M}x{N}x{K}{' silu' if silu else ' +residual'}: {e:.2e}")


def test_fp8_full_path_32k_bitwise_properties():
    """Two layers of the 8B shape, FP8-dynamic, on the benchmark's 32768 tokens: finite logits, identical bit for
    bit for MLP chunks 4096 and 3000 and across repeated runs."""
    w = I.WORKLOADS["llama8b_32k"]
    cfg = w["cfg"].replace(n_layers=2, dtype=I.BF16_FP8)
    tokens = I.make_tokens(cfg, w["tseed"], 32768, request=0)
    cand = I.label_ids(cfg)
    outs = []
    for chunk in (4096, 3000):
        ctx = B.Context(cfg, 32768, chunk)
        try:
            ctx.load_synthetic(w["wseed"], threads=16)
            z, lp = ctx.po_prefill(tokens, cand, want_logits=True)
            if chunk == 4096:
                z2, _ = ctx.po_prefill(tokens, cand, want_logits=True)
                assert np.array_equal(z, z2)
            outs.append(z)
        finally:
            ctx.po_destroy()
    assert np.all(np.isfinite(outs[0])) and np.array_equal(outs[0], outs[1])
