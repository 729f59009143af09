"""Pins for oracle/prefill_oracle.py against things other than itself.

Each pin is chosen so that a plausible slip in the oracle (a dropped term, a wrong sign
or index, a transposed operand, a missing mask or gain) fails at least one of them:
  * scalar brute force of the whole forward pass on tiny inputs (tests/brute_force.py)
  * library routines: torch scaled_dot_product_attention, torch log_softmax, F.silu
  * closed forms for RMSNorm and the rotary embedding
  * attention / SwiGLU special cases with hand-computable answers
  * invariances the paper states: chunk-size independence (Section 4.2), one output
    token from the last position only / causality (Section 1), acceptable-token
    probabilities summing to 1 (Section 2.2)
"""
import math

import numpy as np
import pytest
import torch

from oracle import prefill_oracle as O
from paper_2505_07203_amd import inputs as I
import brute_force as BF
import helpers as H


def micro_cfg(**kw):
    base = dict(n_layers=2, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=8, ffn_dim=24,
                vocab_size=32, rms_eps=1e-5, rope_theta=10000.0, dtype=I.F32, qkv_bias=0)
    base.update(kw)
    return I.ModelConfig(**base)


def micro_weights(cfg, seed, scale=1.0):
    """Weights at micro shapes; `scale` enlarges them so softmax is far from uniform."""
    def grab(kind, layer):
        a = I.stored_to_f64(I.make_tensor(cfg, seed, kind, layer))
        if kind not in I.NORM_KINDS:
            a = a * scale
        return a
    embed = grab(I.KIND_EMBED, -1)
    layers = [{I.KIND_NAMES[k]: grab(k, l) for k in I.layer_kinds(cfg)} for l in range(cfg.n_layers)]
    return embed, layers, grab(I.KIND_FINAL_NORM, -1), grab(I.KIND_LM_HEAD, -1)


# ------------------------------------------------------------------ brute force (whole path)

@pytest.mark.parametrize("bias,hq,hkv", [(0, 4, 2), (1, 4, 2), (0, 4, 4), (0, 4, 1)])
def test_whole_forward_matches_scalar_brute_force(bias, hq, hkv):
    cfg = micro_cfg(qkv_bias=bias, n_q_heads=hq, n_kv_heads=hkv, d_model=16, head_dim=8)
    embed, layers, fnorm, lm = micro_weights(cfg, seed=7, scale=12.0)
    tokens = I.make_tokens(cfg, 11, 9)
    z, _ = O.prefill(tokens, embed, layers, fnorm, lm, cfg)
    xs = O.forward_hidden(tokens, embed, layers, cfg)
    as_lists = [{k: v.tolist() for k, v in W.items()} for W in layers]
    z_bf, x_bf = BF.forward_last_logits([int(t) for t in tokens], embed.tolist(), as_lists,
                                        fnorm.tolist(), lm.tolist(), cfg)
    assert np.max(np.abs(np.array(x_bf) - xs)) < 1e-11
    assert np.max(np.abs(np.array(z_bf) - z)) < 1e-11
    # the test is only meaningful if attention is far from uniform and logits are not tiny
    assert np.max(np.abs(z)) > 0.1


def test_stored_precision_mode_matches_scalar_brute_force():
    """The optional bf16 storage of activations: same rounding points, second implementation."""
    cfg = micro_cfg(qkv_bias=1, n_q_heads=4, n_kv_heads=2, d_model=16, head_dim=8)
    embed, layers, fnorm, lm = micro_weights(cfg, seed=8, scale=12.0)
    tokens = I.make_tokens(cfg, 12, 9)
    z, _ = O.prefill(tokens, embed, layers, fnorm, lm, cfg, store=O.round_bf16)
    xs = O.forward_hidden(tokens, embed, layers, cfg, store=O.round_bf16)
    z_exact, _ = O.prefill(tokens, embed, layers, fnorm, lm, cfg)
    as_lists = [{k: v.tolist() for k, v in W.items()} for W in layers]
    z_bf, x_bf = BF.forward_last_logits([int(t) for t in tokens], embed.tolist(), as_lists,
                                        fnorm.tolist(), lm.tolist(), cfg, store=BF.bf16_scalar)
    assert np.max(np.abs(np.array(x_bf) - xs)) < 1e-11
    assert np.max(np.abs(np.array(z_bf) - z)) < 1e-11
    # the residual stream that comes out is bf16-representable, and the mode is not a no-op
    assert np.array_equal(O.round_bf16(xs), xs)
    assert 1e-4 < np.max(np.abs(z - z_exact)) / np.max(np.abs(z_exact)) < 5e-2
    # store=None and an identity function are the plain definition
    z_id, _ = O.prefill(tokens, embed, layers, fnorm, lm, cfg, store=lambda t: t)
    assert np.array_equal(z_id, z_exact)


def test_round_bf16_matches_torch_and_ties_to_even():
    import torch
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(0, 1, 4096), rng.normal(0, 1e-3, 1024), rng.normal(0, 1e4, 1024),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e38, 1e-40])])
    want = torch.from_numpy(x).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.round_bf16(x)
    assert np.array_equal(got, want)
    # 1 + 2^-8 lies half-way between 1 and 1 + 2^-7: ties go to the even significand (1.0);
    # 1 + 3*2^-8 lies half-way between 1 + 2^-7 and 1 + 2^-6: goes up to the even one
    assert O.round_bf16(np.array([1.00390625]))[0] == 1.0
    assert O.round_bf16(np.array([1.01171875]))[0] == 1.015625
    assert [BF.bf16_scalar(float(v)) for v in x[:512]] == [float(v) for v in got[:512]]


# ------------------------------------------------------------------ library routines

def test_attention_matches_torch_sdpa():
    rng = np.random.default_rng(3)
    N, Hq, Hkv, hd = 37, 6, 2, 16
    q = rng.standard_normal((N, Hq, hd))
    k = rng.standard_normal((N, Hkv, hd))
    v = rng.standard_normal((N, Hkv, hd))
    o = O.causal_gqa_attention(q, k, v)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.from_numpy(v).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0]
    assert np.max(np.abs(ref.permute(1, 0, 2).numpy() - o)) < 1e-12
    # restricted query rows give the same rows
    rows = np.array([0, 5, 36])
    assert np.max(np.abs(O.causal_gqa_attention(q, k, v, rows) - o[rows])) < 1e-14


def test_swiglu_matches_torch_ops():
    rng = np.random.default_rng(4)
    m = rng.standard_normal((5, 12))
    wg, wu, wd = rng.standard_normal((20, 12)), rng.standard_normal((20, 12)), rng.standard_normal((12, 20))
    F = torch.nn.functional
    tm = torch.from_numpy(m)
    ref = F.linear(F.silu(F.linear(tm, torch.from_numpy(wg))) * F.linear(tm, torch.from_numpy(wu)),
                   torch.from_numpy(wd))
    assert np.max(np.abs(ref.numpy() - O.swiglu_mlp(m, wg, wu, wd))) < 1e-12


def test_logprobs_match_torch_log_softmax():
    rng = np.random.default_rng(5)
    z = rng.standard_normal(50) * 4
    cand = np.array([7, 31, 2])
    ref_c = torch.log_softmax(torch.from_numpy(z[cand]), dim=0).numpy()
    assert np.max(np.abs(O.candidate_logprobs(z, cand) - ref_c)) < 1e-13
    ref_f = torch.log_softmax(torch.from_numpy(z), dim=0).numpy()[cand]
    assert np.max(np.abs(O.full_vocab_logprobs(z, cand) - ref_f)) < 1e-13


def test_rmsnorm_matches_torch_rms_norm():
    rng = np.random.default_rng(6)
    x, g = rng.standard_normal((4, 24)), rng.standard_normal(24)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (24,), torch.from_numpy(g), eps=1e-5)
    assert np.max(np.abs(ref.numpy() - O.rmsnorm(x, g, 1e-5))) < 1e-13


# ------------------------------------------------------------------ closed forms: RMSNorm

def test_rmsnorm_closed_forms():
    d, eps = 64, 1e-5
    g = np.linspace(0.5, 1.5, d)
    c = 3.0
    y = O.rmsnorm(np.full(d, c), g, eps)
    assert np.allclose(y, g * c / math.sqrt(c * c + eps), rtol=0, atol=1e-14)
    rng = np.random.default_rng(0)
    x = rng.standard_normal(d)
    ms = float(np.mean(x * x))
    y = O.rmsnorm(x, g, eps)
    assert abs(np.sum((y / g) ** 2) - d * ms / (ms + eps)) < 1e-10
    # scale invariance as eps -> 0
    assert np.max(np.abs(O.rmsnorm(1000 * x, g, 0.0) - O.rmsnorm(x, g, 0.0))) < 1e-12
    # a gain of all ones leaves unit RMS
    assert abs(np.sqrt(np.mean(O.rmsnorm(x, np.ones(d), 0.0) ** 2)) - 1) < 1e-14


# ------------------------------------------------------------------ closed forms: RoPE

def test_rope_closed_forms():
    hd, theta = 16, 10000.0
    rng = np.random.default_rng(1)
    u = rng.standard_normal((6, 3, hd))
    pos = np.arange(6)
    r = O.rope(u, pos, theta)
    assert np.array_equal(r[0], u[0])                                   # t = 0: identity
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(u, axis=-1), atol=1e-13)
    # first pair (0, hd/2) at t=1 rotates by exactly 1 rad; last pair by theta^(-(hd-2)/hd)
    e = np.zeros((2, 1, hd)); e[1, 0, 0] = 1.0
    r1 = O.rope(e, np.array([0, 1]), theta)[1, 0]
    assert abs(r1[0] - math.cos(1.0)) < 1e-15 and abs(r1[hd // 2] - math.sin(1.0)) < 1e-15
    e = np.zeros((2, 1, hd)); e[1, 0, hd // 2 - 1] = 1.0
    a = theta ** (-(hd - 2) / hd)
    r2 = O.rope(e, np.array([0, 1]), theta)[1, 0]
    assert abs(r2[hd // 2 - 1] - math.cos(a)) < 1e-15 and abs(r2[hd - 1] - math.sin(a)) < 1e-15
    # the second component rotates the other way round: (0,1) -> (-sin, cos)
    e = np.zeros((2, 1, hd)); e[1, 0, hd // 2] = 1.0
    r3 = O.rope(e, np.array([0, 1]), theta)[1, 0]
    assert abs(r3[0] + math.sin(1.0)) < 1e-15 and abs(r3[hd // 2] - math.cos(1.0)) < 1e-15
    # relative-position property: <rope(q,m), rope(k,n)> depends on m-n only
    qv, kv = rng.standard_normal((1, 1, hd)), rng.standard_normal((1, 1, hd))
    def ip(m, n):
        return float(np.sum(O.rope(qv, np.array([m]), theta) * O.rope(kv, np.array([n]), theta)))
    assert abs(ip(9, 4) - ip(105, 100)) < 1e-12
    assert abs(ip(9, 4) - ip(4, 9)) > 1e-3                               # and on its sign
    # angles at a long-context position keep full precision
    ang = O.rope_angles(np.array([131071]), 128, 500000.0)[0]
    assert ang[0] == 131071.0
    assert abs(ang[63] - 131071.0 * 500000.0 ** (-126 / 128)) < 1e-12


# ------------------------------------------------------------------ attention special cases

def test_attention_special_cases():
    rng = np.random.default_rng(2)
    N, Hq, Hkv, hd = 12, 4, 2, 8
    q = rng.standard_normal((N, Hq, hd))
    k = rng.standard_normal((N, Hkv, hd))
    v = rng.standard_normal((N, Hkv, hd))
    # N = 1: output is v_0 of the shared kv head
    o1 = O.causal_gqa_attention(q[:1], k[:1], v[:1])
    for h in range(Hq):
        assert np.allclose(o1[0, h], v[0, h // 2], atol=1e-15)
    # q = 0 (or all keys equal): uniform causal average of v
    cm = np.cumsum(v, axis=0) / np.arange(1, N + 1)[:, None, None]
    o0 = O.causal_gqa_attention(np.zeros_like(q), k, v)
    ok = O.causal_gqa_attention(q, np.broadcast_to(k[:1], k.shape), v)
    for h in range(Hq):
        assert np.allclose(o0[:, h], cm[:, h // 2], atol=1e-14)
        assert np.allclose(ok[:, h], cm[:, h // 2], atol=1e-13)
    # the future is masked: changing k, v at positions > t leaves rows <= t unchanged
    k2, v2 = k.copy(), v.copy()
    k2[7:] += 5.0; v2[7:] -= 3.0
    assert np.array_equal(O.causal_gqa_attention(q, k2, v2)[:7], O.causal_gqa_attention(q, k, v)[:7])
    # a very large score on one key selects that key's value (softmax scale sign / max-subtraction)
    qq = np.zeros((N, 1, hd)); kk = np.zeros((N, 1, hd)); vv = rng.standard_normal((N, 1, hd))
    qq[:, 0, 0] = 1e4; kk[3, 0, 0] = 1.0
    ob = O.causal_gqa_attention(qq, kk, vv)
    assert np.allclose(ob[5, 0], vv[3, 0], atol=1e-12) and np.isfinite(ob).all()
    # GQA head mapping is h -> h // G (contiguous groups), checked against per-head MHA
    kr, vr = np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1)
    assert np.allclose(O.causal_gqa_attention(q, kr, vr), O.causal_gqa_attention(q, k, v), atol=1e-15)
    # scale is 1/sqrt(hd): two keys, scores differ by hd -> weights e^{sqrt(hd)} : 1
    q2 = np.ones((2, 1, hd)); k3 = np.zeros((2, 1, hd)); k3[1] = 1.0
    v3 = np.zeros((2, 1, hd)); v3[1] = 1.0
    w = math.exp(math.sqrt(hd)) / (1 + math.exp(math.sqrt(hd)))
    assert abs(O.causal_gqa_attention(q2, k3, v3)[1, 0, 0] - w) < 1e-14


# ------------------------------------------------------------------ block structure

def test_block_special_cases():
    cfg = micro_cfg()
    embed, layers, fnorm, lm = micro_weights(cfg, seed=21, scale=10.0)
    tokens = I.make_tokens(cfg, 5, 7)
    x0 = embed[tokens]
    W = dict(layers[0])
    # Wg = 0 or Wd = 0: the MLP adds nothing; Wo = 0 as well: the block is the identity
    Wz = dict(W, wg=np.zeros_like(W["wg"]), wo=np.zeros_like(W["wo"]))
    assert np.array_equal(O.decoder_layer(x0, Wz, cfg), x0)
    Wz = dict(W, wd=np.zeros_like(W["wd"]), wo=np.zeros_like(W["wo"]))
    assert np.array_equal(O.decoder_layer(x0, Wz, cfg), x0)
    # residual connections: with Wd = 0 the block output is x + attention branch
    Wd0 = dict(W, wd=np.zeros_like(W["wd"]))
    y = O.decoder_layer(x0, Wd0, cfg)
    assert np.max(np.abs(y - x0)) > 1e-3
    # V = 0 kills the attention branch
    Wv0 = dict(W, wv=np.zeros_like(W["wv"]), wd=np.zeros_like(W["wd"]))
    assert np.array_equal(O.decoder_layer(x0, Wv0, cfg), x0)


# ------------------------------------------------------------------ the paper's invariances

def test_chunk_size_invariance():
    """Section 4.2: evaluating the position-wise layers chunk by chunk does not change
    the result."""
    cfg = I.TINY.replace(n_layers=2)
    tokens = I.make_tokens(cfg, 2001, 96)
    z_ref, _ = H.oracle_prefill(cfg, 1001, tokens)
    for c in (1, 7, 64, 96, 1000):
        z, _ = H.oracle_prefill(cfg, 1001, tokens, mlp_chunk=c)
        assert np.max(np.abs(z - z_ref)) < 1e-12


def test_prefix_invariance_and_lazy_last_layer():
    """Causality: the hidden state at position t does not depend on later tokens, so
    prefill(tokens[:t+1]) equals row t of the longer prefill.  Also pins the lazy
    evaluation of the last layer (only its K/V need every position)."""
    cfg = I.TINY.replace(n_layers=2)
    tokens = I.make_tokens(cfg, 2001, 80)
    embed, fnorm, lm = H.oracle_globals(cfg, 1001)
    x_all = O.forward_hidden(tokens, embed, H.oracle_layers(cfg, 1001), cfg)
    for t in (0, 17, 79):
        z_short, _ = H.oracle_prefill(cfg, 1001, tokens[:t + 1])
        z_row = O.last_token_logits(x_all[t], fnorm, lm, cfg.rms_eps)
        assert np.max(np.abs(z_short - z_row)) < 1e-12
    z_lazy, _ = H.oracle_prefill(cfg, 1001, tokens, lazy_last_layer=True)
    z_full, _ = H.oracle_prefill(cfg, 1001, tokens)
    assert np.max(np.abs(z_lazy - z_full)) < 1e-12
    # and it does depend on earlier tokens (the mask is not the wrong way round)
    t2 = tokens.copy(); t2[0] = (t2[0] + 1) % cfg.vocab_size
    z_mod, _ = H.oracle_prefill(cfg, 1001, t2)
    assert np.max(np.abs(z_mod - z_full)) > 1e-6


def test_candidate_probabilities():
    """Section 2.2: the acceptable tokens' probabilities sum to 1."""
    rng = np.random.default_rng(9)
    z = rng.standard_normal(1024) * 3
    cand = np.array([341, 682])
    lp = O.candidate_logprobs(z, cand)
    assert abs(np.sum(np.exp(lp)) - 1) < 1e-15
    assert abs((lp[0] - lp[1]) - (z[341] - z[682])) < 1e-14
    assert np.max(np.abs(O.candidate_logprobs(z + 123.0, cand) - lp)) < 1e-12
    assert abs(np.exp(lp[0]) - 1 / (1 + math.exp(z[682] - z[341]))) < 1e-15


def test_embedding_and_last_row_indexing():
    """Token t reads embedding row tokens[t]; the logits come from the LAST position."""
    cfg = micro_cfg(n_layers=0)
    embed, _, fnorm, lm = micro_weights(cfg, seed=3)
    tokens = np.array([5, 9, 30])
    z, _ = O.prefill(tokens, embed, [], fnorm, lm, cfg)
    xn = embed[30] / math.sqrt(np.mean(embed[30] ** 2) + cfg.rms_eps) * fnorm
    assert np.max(np.abs(z - lm @ xn)) < 1e-15


# ------------------------------------------------------------------ input generator sanity

def test_bf16_rounding_and_streams():
    x = np.array([1.0, 1.00390625, 1.005859375, -2.5, 3.0e-40, 65504.0], dtype=np.float32)
    bits = I.f32_to_bf16_bits(x)
    back = I.bf16_bits_to_f32(bits)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(back, ref)
    # 1.00390625 = 1 + 2^-8 is a tie: rounds to even (1.0); 1.005859375 rounds up to 1 + 2^-7
    assert back[1] == 1.0 and back[2] == 1.0078125
    cfg = I.LLAMA8B.replace(n_layers=1, vocab_size=64)
    a = I.make_tensor(cfg, 1, I.KIND_WQ, 0)
    b = I.make_tensor(cfg, 1, I.KIND_WQ, 0)
    c = I.make_tensor(cfg, 1, I.KIND_WK, 0)
    assert a.dtype == np.uint16 and np.array_equal(a, b)
    assert not np.array_equal(a[:1024], c)
    w = I.bf16_bits_to_f32(a).astype(np.float64)
    assert abs(w.std() - 0.02) < 2e-4 and abs(w.mean()) < 1e-4
    g = I.bf16_bits_to_f32(I.make_tensor(cfg, 1, I.KIND_ATTN_NORM, 0))
    assert abs(g.mean() - 1) < 2e-3 and 0.01 < g.std() < 0.03
    lens = I.workload_lengths("llama8b_mixed16")
    assert len(lens) == 16 and lens.min() >= 256 and lens.max() <= 8192
    t = I.make_tokens(I.LLAMA8B, 2003, 4096)
    assert t.dtype == np.int32 and t.min() >= 0 and t.max() < 128256
