#!/usr/bin/env python3
"""Writes the stored expected values under tests/golden/ for the wide-shape parity cases.

Calls only oracle/ (the float64 definition) and the seeded input generators; nothing here
touches the GPU library.  One JSON file per case holds, for each request, the oracle's
last-token logits at a fixed set of vocabulary ids (evenly spaced ids, the label ids, the
oracle's 16 largest logits) and the candidate log-probs, in two evaluations of the same
definition: "exact" (no activation is rounded) and "stored_bf16" (every tensor kept between
operators is rounded to bfloat16, the storage type of the bf16 workloads; see the oracle's
header).  The file also records what identifies the inputs (config, seeds, lengths, a
SHA-256 of the token ids), so that a GPU test can regenerate the same inputs and compare.

    python tests/golden/make_golden.py --list
    python tests/golden/make_golden.py --case llama8b_L32_N2048 [--case ...]

Layers are the outer loop and requests the inner one, so each layer's weights are generated
once; every request still goes through oracle.decoder_layer unchunked, as defined.
Run time on 8 host cores (both evaluations): about 20 minutes for the 2048-token cases, about
an hour for 2 layers x 32768 tokens; the full 32-layer 32k-token configuration would take
about 14 hours here and has no stored result (the reduced cases stand in for it).
"""
import argparse
import hashlib
import json
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import numpy as np

from oracle import prefill_oracle as O
from paper_2505_07203_amd import inputs as I
import helpers as H

N_EVEN = 509          # evenly spaced sample ids
N_TOP = 16

# case -> (workload whose config and seeds are used, layer count or None for all,
#          request lengths or None for the workload's own, lazy last layer[, "f32"])
# "f32": the same shape and seeds as a float32 model (weights not rounded to bf16; "exact" evaluation only).
# At full depth this is the comparison in which a structural error cannot hide behind the amplified
# bf16 storage noise: the library's float32 path has to match it to a few 1e-4 of the logit range.
CASES = {
    # reduced-cost rungs at full width
    "llama8b_L32_N2048": ("llama8b_32k", None, [2048], False),
    "llama8b_L2_N32768": ("llama8b_32k", 2, [32768], False),
    "llama8b_L8_N32768": ("llama8b_32k", 8, [32768], False),      # a quarter of the benchmark's depth at its full length
    "llama8b_L1_N131072": ("llama8b_128k", 1, [131072], True),
    "qwen32b_L64_N1024": ("qwen32b_8x16k", None, [1024], False),
    "qwen32b_L2_N16384": ("qwen32b_8x16k", 2, [16384], False),
    "qwen32b_L16_N16384": ("qwen32b_8x16k", 16, [16384], False),   # a quarter of the depth at a request's full length
    # a full configuration (16 requests of 256..8192 tokens)
    "llama8b_mixed16": ("llama8b_mixed16", None, None, False),
    # full depth and width in float32
    "llama8b_f32_L32_N2048": ("llama8b_32k", None, [2048], False, "f32"),
    "qwen32b_f32_L64_N1024": ("qwen32b_8x16k", None, [1024], False, "f32"),
}


def sample_ids(V, cand, z):
    even = np.unique(np.round(np.linspace(0, V - 1, N_EVEN)).astype(np.int64))
    top = np.argsort(-z)[:N_TOP]
    return np.unique(np.concatenate([even, np.asarray(cand, dtype=np.int64), top]))


def run_case(name):
    wl, layers, lens, lazy = CASES[name][:4]
    f32 = len(CASES[name]) > 4 and CASES[name][4] == "f32"
    w = I.WORKLOADS[wl]
    cfg = w["cfg"]
    if f32:
        cfg = cfg.replace(dtype=I.F32)
    if layers:
        cfg = cfg.replace(n_layers=layers)
    if lens is None:
        lens = [int(x) for x in I.workload_lengths(wl)]
    cand = I.label_ids(cfg)
    t_all = time.perf_counter()
    reqs = [I.make_tokens(cfg, w["tseed"], n, request=i) for i, n in enumerate(lens)]
    embed = I.make_tensor(cfg, w["wseed"], I.KIND_EMBED, -1)
    modes = {"exact": None} if f32 else {"exact": None, "stored_bf16": O.round_bf16}
    xs = {m: [I.stored_to_f64(embed[t]) for t in reqs] for m in modes}
    del embed
    t_layers = 0.0
    for l in range(cfg.n_layers):
        W = H.oracle_layer(cfg, w["wseed"], l)
        last = lazy and l == cfg.n_layers - 1
        for m, st in modes.items():
            t0 = time.perf_counter()
            xs[m] = [O.decoder_layer(x, W, cfg, None, last_row_only=last, store=st) for x in xs[m]]
            if m == "exact":
                t_layers += time.perf_counter() - t0
        print(f"[{name}] layer {l + 1}/{cfg.n_layers} done, {time.perf_counter() - t_all:.0f} s", flush=True)
        del W
    fnorm = I.stored_to_f64(I.make_tensor(cfg, w["wseed"], I.KIND_FINAL_NORM, -1))
    lm = I.stored_to_f64(I.make_tensor(cfg, w["wseed"], I.KIND_LM_HEAD, -1))
    out_reqs = []
    for i, t in enumerate(reqs):
        rec = {"len": int(len(t)),
               "tokens_sha256": hashlib.sha256(np.ascontiguousarray(t, dtype=np.int32).tobytes()).hexdigest()}
        for m, st in modes.items():
            z = O.last_token_logits(xs[m][i][-1], fnorm, lm, cfg.rms_eps, store=st)
            lp = O.candidate_logprobs(z, cand)
            ids = sample_ids(cfg.vocab_size, cand, z)
            order = np.argsort(-z)
            rec[m] = {
                "argmax": int(order[0]),
                "top_gap": float(z[order[0]] - z[order[1]]),
                "max_abs_logit": float(np.max(np.abs(z))),
                "sample_ids": [int(j) for j in ids],
                "sample_logits": [float(np.float32(z[j])) for j in ids],
                "top_ids": [int(j) for j in order[:N_TOP]],
                "cand_logprobs": [float(v) for v in lp],
            }
        out_reqs.append(rec)
    doc = {
        "kind": "prefill_last_token_logits",
        "source": "oracle/prefill_oracle.py (float64), written by tests/golden/make_golden.py",
        "citation": "Section 4.2: chunked position-wise layers leave the result unchanged; "
                    "Section 2.2: acceptable-token probabilities sum to 1",
        "case": name, "workload": wl, "layers": cfg.n_layers, "lazy_last_layer": bool(lazy),
        "model_dtype": "f32" if f32 else "bf16",
        "wseed": w["wseed"], "tseed": w["tseed"], "mlp_chunk": w["chunk"],
        "cand_ids": [int(c) for c in cand],
        "oracle_layer_seconds_exact_mode": t_layers, "oracle_total_seconds": time.perf_counter() - t_all,
        "host_cores": os.cpu_count(),
        "requests": out_reqs,
    }
    path = os.path.join(HERE, name + ".json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=0)
        f.write("\n")
    print(f"[{name}] wrote {path} ({doc['oracle_total_seconds']:.0f} s)", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--case", action="append", default=[])
    ap.add_argument("--list", action="store_true")
    a = ap.parse_args()
    if a.list or not a.case:
        for k, v in CASES.items():
            print(k, v)
        return
    for c in a.case:
        run_case(c)


if __name__ == "__main__":
    main()
