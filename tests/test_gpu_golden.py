"""Wide-shape parity: libpo against stored float64-oracle results (tests/golden/*.json).

Each file was written by tests/golden/make_golden.py from oracle/ alone and holds two
evaluations of the definition: "exact" (nothing rounded) and "stored_bf16" (every tensor kept
between operators rounded to bfloat16, as a bf16 model stores them).  The inputs are
regenerated here from the recorded seeds (and checked against the recorded SHA-256 of the
token ids), run through po_prefill at the recorded chunk size, and compared at the stored
vocabulary ids.

Bar (bf16 path), with err(a, b) = max|a - b| / max|oracle logit over the vocabulary|:
  err(GPU, stored_bf16) <= tol and err(GPU, exact) <= tol, the same top-1 token, the same
  preferred label, the label log-prob difference within tol * max|oracle|, where
  tol = max(2e-2, 2 * err(stored_bf16, exact)).
Why the second term: a deep randomly initialised decoder amplifies every 2^-9 rounding of a
stored activation (no trained structure damps it).  At 2 layers the oracle's two evaluations
differ by a few 1e-3 and tol is the plain 2e-2; at 32 layers they differ from EACH OTHER by
4.6e-2 of the logit range, although both are float64 evaluations of the same definition, so no
bf16-storing implementation can be expected within 2e-2 of either.  That distance is measured
by the oracle alone (no GPU value enters it), and the GPU path may not be further from either
evaluation than twice it.  The per-operator tests in test_gpu_parity.py hold every kernel to
its tight, un-amplified tolerance at the same widths.

Requests of up to 2048 tokens are also run in few-rows mode (po_set_few_rows_split) and held to the
same bar: that mode sums in another order, so it is compared with the oracle, not with the default path.

Top-1 rule: when the oracle's own gap between its two largest logits is below the error the
tolerance allows (2 * 2e-2 * max|oracle|) several answers are correct; then the GPU's
top-1 only has to be one of the oracle's 16 largest whose logit lies within that margin.
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


def _check_block(case, i, z, lp, block, tol):
    scale = block["max_abs_logit"]
    err = _err(z, block)
    assert err <= tol, (case, i, err, tol)
    top = int(np.argmax(z))
    if block["top_gap"] >= 2 * tol * scale:
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


@pytest.mark.parametrize("path", GOLDEN, ids=[os.path.basename(p)[:-5] for p in GOLDEN])
def test_against_stored_oracle(path):
    from paper_2505_07203_amd import binding as B
    doc = _load(path)
    if doc.get("kind") != "prefill_last_token_logits":
        pytest.skip("not a logits fixture")
    w = I.WORKLOADS[doc["workload"]]
    assert (w["wseed"], w["tseed"]) == (doc["wseed"], doc["tseed"])
    cfg = w["cfg"].replace(n_layers=doc["layers"])
    cand = doc["cand_ids"]
    lens = [r["len"] for r in doc["requests"]]
    ctx = B.Context(cfg, max(lens), doc["mlp_chunk"])
    try:
        ctx.load_synthetic(doc["wseed"], threads=16)
        singles = []
        for i, r in enumerate(doc["requests"]):
            t = I.make_tokens(cfg, doc["tseed"], r["len"], request=i)
            assert hashlib.sha256(np.ascontiguousarray(t, dtype=np.int32).tobytes()).hexdigest() == r["tokens_sha256"]
            z, lp = ctx.po_prefill(t, cand, want_logits=True)
            assert abs(float(np.sum(np.exp(lp.astype(np.float64)))) - 1.0) < 1e-5
            ex, sb = r["exact"], r["stored_bf16"]
            # what storing activations in bf16 costs by itself, from the oracle's two evaluations
            common = sorted(set(ex["sample_ids"]) & set(sb["sample_ids"]))
            e_by, s_by = dict(zip(ex["sample_ids"], ex["sample_logits"])), dict(zip(sb["sample_ids"], sb["sample_logits"]))
            storage_dev = max(abs(e_by[j] - s_by[j]) for j in common) / ex["max_abs_logit"]
            tol = max(TOL, 2 * storage_dev)
            err_s = _check_block(doc["case"], i, z, lp, sb, tol)
            err_e = _check_block(doc["case"], i, z, lp, ex, tol)
            print(f"{doc['case']} request {i} len {r['len']}: err vs stored_bf16 {err_s:.3e}, vs exact {err_e:.3e} "
                  f"(oracle stored-vs-exact {storage_dev:.3e}, tol {tol:.3e})")
            singles.append((z, lp))
            if r["len"] <= 2048:
                # few-rows mode (split reductions, another summation order): the same bar against the oracle
                ctx.po_set_few_rows_split(True)
                zs, lps = ctx.po_prefill(t, cand, want_logits=True)
                assert ctx.po_get_stats()["split_launches"] > 0
                ctx.po_set_few_rows_split(False)
                err_ss = _check_block(doc["case"], i, zs, lps, sb, tol)
                err_se = _check_block(doc["case"], i, zs, lps, ex, tol)
                print(f"    few-rows mode: err vs stored_bf16 {err_ss:.3e}, vs exact {err_se:.3e}")
        if len(singles) > 1:
            # the same requests with their position-wise layers packed: the same bits, request by request
            toks = [I.make_tokens(cfg, doc["tseed"], r["len"], request=i) for i, r in enumerate(doc["requests"])]
            zp, lpp = ctx.po_prefill_packed(toks, cand, want_logits=True)
            for i, (z, lp) in enumerate(singles):
                assert np.array_equal(zp[i], z) and np.array_equal(lpp[i], lp), (doc["case"], i)
    finally:
        ctx.po_destroy()
