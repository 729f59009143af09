"""Wide-shape parity: libpo against stored float64-oracle results (tests/golden/*.json).

Each file was written by tests/golden/make_golden.py from oracle/ alone and holds two
evaluations of the definition: "exact" (nothing rounded) and "stored_bf16" (every tensor kept
between operators rounded to bfloat16, as a bf16 model stores them).  The inputs are
regenerated here from the recorded seeds (and checked against the recorded SHA-256 of the
token ids), run through po_prefill at the recorded chunk size, and compared at the stored
vocabulary ids.

Bar (bf16 path), with err(a, b) = max|a - b| / max|oracle logit over the vocabulary|:
  err(GPU, stored_bf16) <= tol and err(GPU, exact) <= tol, the same preferred label, the label
  log-prob difference within tol * max|oracle|, where tol = max(2e-2, 1.5 * err(stored_bf16, exact)).
Why the second term: a deep randomly initialised decoder amplifies every 2^-9 rounding of a
stored activation (no trained structure damps it).  At 2 layers the oracle's two evaluations
differ by a few 1e-3 and tol is the plain 2e-2; at 32 layers they differ from EACH OTHER by
4.6e-2 of the logit range, although both are float64 evaluations of the same definition, so no
bf16-storing implementation can be expected within 2e-2 of either.  That distance is measured
by the oracle alone (no GPU value enters it).  For one request it is one draw of the amplified noise
and so is the GPU's distance; in a fixture with several requests of the same depth the reference
distance of a request is therefore its own or the fixture's median, whichever is larger (on the
16-request fixture the draws range over 2.8 .. 5.4e-2 and the GPU's over 3.0 .. 4.9e-2).  The GPU path
may not be further than 1.5 times that from either evaluation.  The per-operator tests in
test_gpu_parity.py hold every kernel to its tight, un-amplified tolerance at the same widths.

Bar (float32 fixtures, "model_dtype": "f32": the same shapes, depths and seeds run as a float32
model, "exact" evaluation only): err(GPU, exact) <= 1e-3 and the same top-1 token, always.  This is
the comparison at full depth and width in which nothing is amplified beyond float32 rounding, so a
structural error at depth (a wrong layer's weights, a stale buffer, a wrong position) cannot hide
in the bf16 margin above.

Top-1 rule (bf16 fixtures).  Requests are screened with the ORACLE alone: a request whose gap
between its two largest logits is at least 5 % of max|logit| in both evaluations, with the same
top-1 in both, has one right answer whatever the rounding, and the GPU must give exactly it.  The
other requests (random-init logits over a vocabulary of 128 k have close leaders) are screened out
of the strict rule and say so in the log; for them the GPU's top-1 must still be a token whose
oracle logit lies within the error the tolerance allows of the oracle's largest, which is what the
error bound implies and no more.

Requests of up to 2048 tokens are also run in few-rows mode (po_set_few_rows_split) and held to the
same bar: that mode sums in another order, so it is compared with the oracle, not with the default path.
"""
import glob
import hashlib
import json
import os

import numpy as np
import pytest

from paper_2505_07203_amd import inputs as I

pytestmark = pytest.mark.gpu

GOLDEN = sorted(glob.glob(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "*.json")))
TOL = 2e-2


def _load(path):
    with open(path) as f:
        return json.load(f)


def _err(z, block):
    ids = np.asarray(block["sample_ids"])
    ref = np.asarray(block["sample_logits"], dtype=np.float64)
    return float(np.max(np.abs(z[ids].astype(np.float64) - ref)) / block["max_abs_logit"])


SCREEN_GAP = 0.05      # oracle-only screen for the strict top-1 rule: gap of the two largest logits / max|logit|
STORAGE_FACTOR = 1.5   # the GPU path may be this many times the oracle's own stored-vs-exact distance away
TOL_F32 = 1e-3
# float32 path with storage rounding against the oracle's stored_bf16 evaluation: the two round the same tensors at the
# same points, but rounding is discontinuous, so float32 against float64 arithmetic before a rounding flips bf16 codes,
# and through a deep stack the two realisations drift apart (measured: 2e-3 .. 4e-3 on 1-2 layers, half the storage
# effect itself on 32 / 64 layers).  Bar: 1e-2, or closer to each other than either is to the unrounded result.
TOL_F32_STORED = 1e-2


def _check_block(case, i, z, lp, block, tol, strict_top1):
    scale = block["max_abs_logit"]
    err = _err(z, block)
    assert err <= tol, (case, i, err, tol)
    top = int(np.argmax(z))
    if strict_top1:
        assert top == block["argmax"], (case, i, top, block["argmax"])
    else:
        ref_by_id = dict(zip(block["sample_ids"], block["sample_logits"]))
        ok = [j for j in block["top_ids"] if ref_by_id[block["argmax"]] - ref_by_id[j] <= 2 * tol * scale]
        assert top in ok, (case, i, top, ok)
    ref_lp = np.asarray(block["cand_logprobs"])
    assert abs((lp[0] - lp[1]) - (ref_lp[0] - ref_lp[1])) <= tol * scale
    if abs(ref_lp[0] - ref_lp[1]) > 2 * tol * scale:
        assert int(np.argmax(lp)) == int(np.argmax(ref_lp))
    return err


def _screen(r):
    """The oracle-only screen: one right top-1 whatever the rounding."""
    ex, sb = r["exact"], r["stored_bf16"]
    return (ex["argmax"] == sb["argmax"] and ex["top_gap"] >= SCREEN_GAP * ex["max_abs_logit"]
            and sb["top_gap"] >= SCREEN_GAP * sb["max_abs_logit"])


@pytest.mark.parametrize("path", GOLDEN, ids=[os.path.basename(p)[:-5] for p in GOLDEN])
def test_against_stored_oracle(path):
    from paper_2505_07203_amd import binding as B
    doc = _load(path)
    if doc.get("kind") != "prefill_last_token_logits":
        pytest.skip("not a logits fixture")
    w = I.WORKLOADS[doc["workload"]]
    assert (w["wseed"], w["tseed"]) == (doc["wseed"], doc["tseed"])
    cfg = w["cfg"].replace(n_layers=doc["layers"])
    f32 = doc.get("model_dtype") == "f32"
    if f32:
        cfg = cfg.replace(dtype=I.F32)
    cand = doc["cand_ids"]
    lens = [r["len"] for r in doc["requests"]]
    ctx = B.Context(cfg, max(lens), doc["mlp_chunk"])
    # single-request bf16 fixtures are also run through the float32 path (below): its context is loaded alongside,
    # from the same generated tensors
    ctx32 = None
    if not f32 and len(doc["requests"]) == 1:
        ctx32 = B.Context(cfg.replace(dtype=I.F32), max(lens), doc["mlp_chunk"])
    try:
        B.load_synthetic_models([ctx] + ([ctx32] if ctx32 else []), doc["wseed"], threads=16)
        singles = []

        def _storage_dev(r):
            # what storing activations in bf16 costs by itself, from the oracle's two evaluations
            ex, sb = r["exact"], r["stored_bf16"]
            e_by, s_by = dict(zip(ex["sample_ids"], ex["sample_logits"])), dict(zip(sb["sample_ids"], sb["sample_logits"]))
            return max(abs(e_by[j] - s_by[j]) for j in set(e_by) & set(s_by)) / ex["max_abs_logit"]
        dev_median = 0.0 if f32 else float(np.median([_storage_dev(r) for r in doc["requests"]]))
        for i, r in enumerate(doc["requests"]):
            t = I.make_tokens(cfg, doc["tseed"], r["len"], request=i)
            assert hashlib.sha256(np.ascontiguousarray(t, dtype=np.int32).tobytes()).hexdigest() == r["tokens_sha256"]
            z, lp = ctx.po_prefill(t, cand, want_logits=True)
            assert abs(float(np.sum(np.exp(lp.astype(np.float64)))) - 1.0) < 1e-5
            if f32:
                err_e = _check_block(doc["case"], i, z, lp, r["exact"], TOL_F32, True)
                print(f"{doc['case']} request {i} len {r['len']}: float32 path vs exact {err_e:.3e} (tol {TOL_F32:.0e}), "
                      f"top-1 {int(np.argmax(z))} == {r['exact']['argmax']}, oracle gap "
                      f"{r['exact']['top_gap'] / r['exact']['max_abs_logit']:.2e} of the range")
                continue
            ex, sb = r["exact"], r["stored_bf16"]
            storage_dev = _storage_dev(r)
            tol = max(TOL, STORAGE_FACTOR * max(storage_dev, dev_median))
            strict = _screen(r)
            err_s = _check_block(doc["case"], i, z, lp, sb, tol, strict)
            err_e = _check_block(doc["case"], i, z, lp, ex, tol, strict)
            print(f"{doc['case']} request {i} len {r['len']}: err vs stored_bf16 {err_s:.3e}, vs exact {err_e:.3e} "
                  f"(oracle stored-vs-exact {storage_dev:.3e}, tol {tol:.3e}; "
                  f"{'strict top-1' if strict else 'screened out of the strict top-1 rule by the oracle: leaders too close'})")
            singles.append((z, lp))
            if r["len"] <= 2048:
                # few-rows mode (split reductions, another summation order): the same bar against the oracle
                ctx.po_set_few_rows_split(True)
                zs, lps = ctx.po_prefill(t, cand, want_logits=True)
                assert ctx.po_get_stats()["split_launches"] > 0
                ctx.po_set_few_rows_split(False)
                err_ss = _check_block(doc["case"], i, zs, lps, sb, tol, strict)
                err_se = _check_block(doc["case"], i, zs, lps, ex, tol, strict)
                print(f"    few-rows mode: err vs stored_bf16 {err_ss:.3e}, vs exact {err_se:.3e}")
        if len(singles) > 1:
            # the same requests with their position-wise layers packed: the same bits, request by request
            toks = [I.make_tokens(cfg, doc["tseed"], r["len"], request=i) for i, r in enumerate(doc["requests"])]
            zp, lpp = ctx.po_prefill_packed(toks, cand, want_logits=True)
            for i, (z, lp) in enumerate(singles):
                assert np.array_equal(zp[i], z) and np.array_equal(lpp[i], lp), (doc["case"], i)
    except BaseException:
        if ctx32:
            ctx32.po_destroy()
        raise
    finally:
        ctx.po_destroy()
    if ctx32:
        # The float32 path in its two evaluation modes against the oracle's two evaluations of the same fixture: nothing
        # rounded against "exact", every tensor kept between operators rounded to bf16 (po_set_storage_rounding)
        # against "stored_bf16".  This anchors test_gpu_fullconfig.py, where the same two modes stand in for the
        # oracle at configurations no float64 CPU run reaches, at full depth (2048 / 1024 tokens) and at full length
        # (32768, 131072, 16384 tokens on 1-2 layers).  The context holds the bf16 model's weight values.
        ctx = ctx32
        try:
            r = doc["requests"][0]
            t = I.make_tokens(cfg, doc["tseed"], r["len"], request=0)
            z, lp = ctx.po_prefill(t, cand, want_logits=True)
            err_e = _check_block(doc["case"], 0, z, lp, r["exact"], TOL_F32, _screen(r))
            ctx.po_set_storage_rounding(True)
            z, lp = ctx.po_prefill(t, cand, want_logits=True)
            tol_s = max(TOL_F32_STORED, _storage_dev(r))
            err_s = _check_block(doc["case"], 0, z, lp, r["stored_bf16"], tol_s, _screen(r))
            print(f"    float32 path, the same fixture: vs exact {err_e:.3e} (tol {TOL_F32:.0e}); with bf16 storage rounding "
                  f"vs stored_bf16 {err_s:.3e} (tol {tol_s:.1e})")
        finally:
            ctx.po_destroy()
