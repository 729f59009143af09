"""Few-rows mode (po_set_few_rows_split): requests that compute few positions -- short ones, or the
suffix behind a long cached prefix -- run their narrow GEMMs split over K and their attention split over
the keys.  Sums are formed in another order than on the default path, so the bar is the one every bf16
result meets: within 2e-2 of the float64 oracle (normalised by the logit range) with the oracle's top-1
and preferred label; plus closeness to the default path's own result, and bit-identity between repeated
runs (the partial sums are added in a fixed order, no atomics)."""
import numpy as np
import pytest

from paper_2505_07203_amd import inputs as I
from tests import helpers as H

pytestmark = pytest.mark.gpu

# widths chosen so that every split kernel engages at the tiny shape: K of the O-projection / QKV = 256
# (4 slices -> 2 splits), of the down projection = 768 (12 slices -> 4 splits); head dimension 64
TINY_BF16 = I.TINY.replace(dtype=I.BF16, ffn_dim=768)


def _ctx(cfg, wseed, max_len, chunk):
    from paper_2505_07203_amd import binding as B
    ctx = B.Context(cfg, max_len, chunk)
    ctx.load_synthetic(wseed, threads=4)
    return ctx


def _screened(cfg, wseed, tseed, n, min_gap=0.05):
    """First token seed whose ORACLE logits have a clear top-1 (no GPU value involved)."""
    for k in range(8):
        t = I.make_tokens(cfg, tseed + 1000 * k, n)
        z, _ = H.oracle_prefill(cfg, wseed, t)
        top2 = np.sort(z)[-2:]
        if top2[1] - top2[0] >= min_gap * np.max(np.abs(z)):
            return t, z
    raise AssertionError("no screened seed")


@pytest.mark.parametrize("n", [40, 150, 256, 600])
def test_short_request_against_oracle(n):
    cfg = TINY_BF16
    tokens, ref = _screened(cfg, 31, 500 + n, n)
    cand = I.label_ids(cfg)
    ctx = _ctx(cfg, 31, 1024, 512)
    try:
        z0, lp0 = ctx.po_prefill(tokens, cand)
        ctx.po_set_few_rows_split(True)
        z1, lp1 = ctx.po_prefill(tokens, cand)
        z2, lp2 = ctx.po_prefill(tokens, cand)
        assert np.array_equal(z1, z2) and np.array_equal(lp1, lp2)              # deterministic
        for z in (z0, z1):
            rel = H.normalised_max_rel(z, ref)
            assert rel <= 2e-2, rel
            assert int(np.argmax(z)) == int(np.argmax(ref))
            assert int(np.argmax(z[cand])) == int(np.argmax(ref[cand]))
        assert H.normalised_max_rel(z1, z0) <= 1e-2
        assert abs(float(np.sum(np.exp(lp1.astype(np.float64)))) - 1.0) < 1e-5
        assert ctx.po_get_stats()["split_launches"] > 0                          # the split kernels did run
        ctx.po_set_few_rows_split(False)
        ctx.po_prefill(tokens, cand)
        assert ctx.po_get_stats()["split_launches"] == 0
    finally:
        ctx.po_destroy()


@pytest.mark.parametrize("prefix,suffix", [(700, 100), (512, 1), (300, 257), (1000, 24)])
def test_suffix_behind_cached_prefix_against_oracle(prefix, suffix):
    cfg = TINY_BF16
    n = prefix + suffix
    tokens, ref = _screened(cfg, 32, 900 + n, n)
    cand = I.label_ids(cfg)
    ctx = _ctx(cfg, 32, 1024, 512)
    try:
        z0, _ = ctx.po_prefill(tokens, cand)
        ctx.po_attach_kv_cache(1024)
        ctx.po_prefill_prefix(tokens, prefix, cand)                              # stores the prefix (default path)
        ctx.po_set_few_rows_split(True)
        z1, lp1, reused = ctx.po_prefill_prefix(tokens, 0, cand)
        assert reused == prefix
        rel = H.normalised_max_rel(z1, ref)
        assert rel <= 2e-2, rel
        assert int(np.argmax(z1)) == int(np.argmax(ref))
        assert int(np.argmax(z1[cand])) == int(np.argmax(ref[cand]))
        assert H.normalised_max_rel(z1, z0) <= 1e-2
        assert ctx.po_get_stats()["split_launches"] > 0
        # a prefix stored in this mode serves the default path and the other way round
        ctx.po_attach_kv_cache(1024)
        ctx.po_prefill_prefix(tokens, prefix, cand)
        ctx.po_set_few_rows_split(False)
        z2, _, reused = ctx.po_prefill_prefix(tokens, 0, cand)
        assert reused == prefix and H.normalised_max_rel(z2, ref) <= 2e-2
    finally:
        ctx.po_destroy()


def test_full_width_two_layers_against_default_path():
    """8B widths (d 4096, 32 / 8 heads of 128, F 14336), two layers: the split kernels at the shapes the
    serving trace runs them at, against the default path (itself held to the oracle elsewhere)."""
    cfg = I.LLAMA8B.replace(n_layers=2, vocab_size=4096)
    cand = I.label_ids(cfg)
    ctx = _ctx(cfg, 7, 10240, 4096)
    try:
        for prefix, suffix in ((9000, 150), (4000, 300), (0, 200), (8192, 1000)):
            t = I.make_tokens(cfg, 5 + prefix, prefix + suffix)
            ctx.po_set_few_rows_split(False)
            ref, ref_lp = ctx.po_prefill(t, cand)
            ctx.po_attach_kv_cache(10240)
            if prefix:
                ctx.po_prefill_prefix(t, prefix, cand, want_logits=False)
            ctx.po_set_few_rows_split(True)
            z, lp, reused = ctx.po_prefill_prefix(t, 0, cand)
            assert reused == prefix
            rel = H.normalised_max_rel(z, ref)
            print(f"prefix {prefix} suffix {suffix}: split vs default {rel:.3e}")
            assert rel <= 2e-2 and int(np.argmax(z)) == int(np.argmax(ref))
            assert abs((lp[0] - lp[1]) - (ref_lp[0] - ref_lp[1])) <= 2e-2 * float(np.max(np.abs(ref)))
    finally:
        ctx.po_destroy()


def test_packed_short_requests_in_few_rows_mode():
    cfg = TINY_BF16
    cand = I.label_ids(cfg)
    lens = [300, 90, 512, 40]
    toks = [I.make_tokens(cfg, 77, n, request=i) for i, n in enumerate(lens)]
    ctx = _ctx(cfg, 33, 1024, 512)
    try:
        ref = [ctx.po_prefill(t, cand) for t in toks]
        ctx.po_set_few_rows_split(True)
        zp, lpp = ctx.po_prefill_packed(toks, cand, want_logits=True)
        for i, (z, lp) in enumerate(ref):
            assert H.normalised_max_rel(zp[i], z) <= 1e-2, i
            assert int(np.argmax(zp[i])) == int(np.argmax(z))
    finally:
        ctx.po_destroy()


@pytest.mark.parametrize("M,N,K", [(150, 4096, 4096), (1, 4096, 14336), (32, 256, 2048), (256, 512, 4096), (100, 320, 1024),
                                   (600, 4096, 4096), (257, 1024, 14336), (2000, 4096, 4096)])
def test_split_linear_against_float64(M, N, K):
    """The split-K residual GEMM by itself: C = A W^T + R against numpy float64 on the stored bf16 operands.
    Bar: the fp32 accumulation error of K products plus ONE bf16 rounding of the result, as for po_op_linear."""
    import torch
    from paper_2505_07203_amd import binding as B
    g = torch.Generator(device="cpu").manual_seed(M * 7 + N + K)
    a = torch.randn(M, K, generator=g).to(torch.bfloat16).cuda()
    w = (torch.randn(N, K, generator=g) * 0.05).to(torch.bfloat16).cuda()
    r = torch.randn(M, N, generator=g).to(torch.bfloat16).cuda()
    c, splits = B.po_op_linear_split(a, w, r)
    assert splits >= 2 and c is not None, "this shape was meant to split"
    ref = a.double().cpu().numpy() @ w.double().cpu().numpy().T + r.double().cpu().numpy()
    got = c.double().cpu().numpy()
    tol = 2.0 ** -8 * np.abs(ref) + 1e-5 * K ** 0.5 * np.max(np.abs(ref))      # half an ulp of bf16, plus accumulation
    assert np.all(np.abs(got - ref) <= tol), float(np.max(np.abs(got - ref) - tol))
    # the unsplit kernel on the same operands: equal up to the rounding of the summation order
    c0 = B.po_op_linear(a, w, residual=r)
    d = (c.double() - c0.double()).abs().cpu().numpy()
    assert np.all(d <= 2.0 ** -7 * np.abs(ref) + 2e-5 * K ** 0.5 * np.max(np.abs(ref))), float(d.max())


def test_split_linear_declines_large_shapes():
    import torch
    from paper_2505_07203_amd import binding as B
    a = torch.zeros(4096, 4096, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(4096, 4096, dtype=torch.bfloat16, device="cuda")
    r = torch.zeros(4096, 4096, dtype=torch.bfloat16, device="cuda")
    c, splits = B.po_op_linear_split(a, w, r)
    assert c is None and splits <= 1                        # 256 tiles fill the chip: nothing to split
    a = torch.zeros(64, 4096, dtype=torch.bfloat16, device="cuda")
    c, splits = B.po_op_linear_split(a, w, r[:64].contiguous(), scratch_bytes=4096)
    assert c is None and splits <= 1                        # scratch too small for even two planes


@pytest.mark.parametrize("N,q_row0,Hq,Hkv,hd", [(600, 450, 4, 2, 64), (1500, 1499, 8, 2, 128), (2000, 1000, 8, 2, 128),
                                                 (4097, 4000, 5, 1, 128), (700, 0, 4, 4, 64), (3000, 2900, 32, 8, 128)])
def test_split_attention_against_float64(N, q_row0, Hq, Hkv, hd):
    """The split-key attention by itself: rows [q_row0, N) against the oracle's plain causal GQA attention."""
    import torch
    from oracle import prefill_oracle as O
    from paper_2505_07203_amd import binding as B
    rng = np.random.default_rng(N + q_row0)
    def stored(shape, scale=1.0):
        return I.f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))
    q, k, v = stored((N, Hq, hd)), stored((N, Hkv, hd)), stored((N, Hkv, hd))
    dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    o, splits = B.po_op_attention_split(dev(q), dev(k), dev(v), q_row0)
    assert splits >= 2 and o is not None, "this shape was meant to split"
    ref = O.causal_gqa_attention(I.stored_to_f64(q), I.stored_to_f64(k), I.stored_to_f64(v))[q_row0:]
    got = o[q_row0:].double().cpu().numpy()
    err = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
    print(f"split attention N={N} rows from {q_row0} Hq={Hq} Hkv={Hkv} hd={hd} splits={splits}: {err:.3e}")
    assert err <= 1.5e-2
    assert not o[:q_row0].any()                      # rows below q_row0 untouched
