"""CPU oracle for the single-output-token prefill forward pass.  TEST INFRASTRUCTURE ONLY.

This file is the plain definition of what the hot path computes, written out in float64
numpy with no chunking, no KV-buffer reuse, no online softmax and no tiling: the paper's
method reaches exactly the textbook result (Section 4.2: chunking the position-wise
layers does not change the inference result; Section 1/abstract: the KV cache of earlier
layers is dead because nothing is decoded), so the oracle *is* that textbook result.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import it.  It
shares no code with the HIP library and imports nothing from the product package.

What each function follows:
  * prefill / one output token / acceptable-token list     -- Section 1 (prefill-only
    workloads, footnote on the acceptable-token list), Section 2.2 (P(Yes)+P(No)=1)
  * MLP structure gate/up/down with 2F intermediates/token -- Section 4.1 (28672 numbers
    per token for Llama-3.1-8B = 2 x 14336) and its MLP figure
  * chunk-by-chunk evaluation of position-wise layers      -- Section 4.2 / 4.3 (optional
    `mlp_chunk` argument; used only to pin the invariance, never needed for the result)
The decoder architecture itself (pre-norm block, RMSNorm, rotary embedding with the
rotate-half pairing (i, i+hd/2), grouped-query attention, SwiGLU, untied LM head) is not
defined by the paper; it is the Llama family's published architecture named by the
workload configs.

Parity status: every function here is pinned by tests/test_oracle_pins.py (brute-force
scalar evaluation on tiny inputs, library routines, closed forms, invariances).  Outputs
at the full 8B/32B shapes are "parity unpinned by the paper": the paper prints no logits;
they are pinned only through the same code being pinned at small shapes.

Weights are passed as float64 arrays holding the *stored* values (bf16-rounded for bf16
models; exactly representable).  Matrix layout is the checkpoint convention
[out_features, in_features]; y = x @ W.T.

Storage precision of activations.  By default nothing is rounded: every activation stays in
float64 ("exact" mode).  A bf16 model also *stores* its activations in bf16, and a 32-layer
randomly initialised decoder amplifies each such rounding (2^-9 relative) to a few percent
of the logit range whatever the implementation -- measured with this file alone by
comparing the two modes.  The optional `store` argument (a function array -> array, e.g.
`round_bf16`) is applied to every tensor the forward pass materialises between operators:
the two normalised activations, Q and K after the rotary embedding, V, the attention
output, the SiLU-gated MLP intermediate, and the residual stream after each of its two
updates.  All arithmetic inside an operator (dot products, softmax, norms) stays float64.
With `store=None` the functions are the plain definition.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "round_bf16", "rmsnorm", "rope_angles", "rope", "causal_gqa_attention", "swiglu_mlp",
    "decoder_layer", "forward_hidden", "last_token_logits", "candidate_logprobs",
    "full_vocab_logprobs", "prefill",
]


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 (8 significand bits, float32 exponent range), ties to even,
    returned as float64.  The value is first rounded to float32 (ties to even), then the
    low 16 bits of the float32 pattern are rounded away."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32).reshape(f.shape).astype(np.float64)


def _keep(t):
    return t


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y_j = x_j * g_j / sqrt(mean_k x_k^2 + eps), over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)


def rope_angles(positions: np.ndarray, head_dim: int, theta: float) -> np.ndarray:
    """angle[t, i] = t * theta^(-2i/head_dim), i = 0 .. head_dim/2 - 1 (float64)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = np.float64(theta) ** (-2.0 * i / head_dim)
    return np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]


def rope(u: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding, rotate-half pairing: for each head vector u[t, h, :]
    the pair (u_i, u_{i+hd/2}) is rotated by angle[t, i].
    u: [N, H, hd] -> [N, H, hd]."""
    u = np.asarray(u, dtype=np.float64)
    hd = u.shape[-1]
    half = hd // 2
    ang = rope_angles(positions, hd, theta)          # [N, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def causal_gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray,
                         query_rows: np.ndarray | None = None) -> np.ndarray:
    """o[t, h] = sum_{s<=t} softmax_s(q[t,h].k[s,h//G] / sqrt(hd)) v[s,h//G].

    q: [N, Hq, hd]; k, v: [N, Hkv, hd]; G = Hq // Hkv.  Two-pass softmax over the
    explicitly masked score row.  `query_rows` (optional) restricts the evaluated query
    positions (each still attends to all keys s <= t); the result then has that many
    rows.  Returns [rows, Hq, hd]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    N, Hq, hd = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    rows = np.arange(N) if query_rows is None else np.asarray(query_rows, dtype=np.int64)
    out = np.empty((len(rows), Hq, hd), dtype=np.float64)
    scale = 1.0 / np.sqrt(np.float64(hd))
    key_pos = np.arange(N)
    # rows are processed in groups only to bound the memory of the score matrix;
    # every row is the full definition.
    step = max(1, min(len(rows), (1 << 24) // max(N, 1)))
    for h in range(Hq):
        c = h // G
        kc, vc = k[:, c, :], v[:, c, :]
        for r0 in range(0, len(rows), step):
            rr = rows[r0:r0 + step]
            s = (q[rr, h, :] @ kc.T) * scale                     # [rows, N]
            s = np.where(key_pos[None, :] <= rr[:, None], s, -np.inf)
            m = np.max(s, axis=1, keepdims=True)
            p = np.exp(s - m)
            p = p / np.sum(p, axis=1, keepdims=True)
            out[r0:r0 + step, h, :] = p @ vc
    return out


def _matmul_t(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    return x @ w.T


def swiglu_mlp(m: np.ndarray, wg: np.ndarray, wu: np.ndarray, wd: np.ndarray, store=None, linear=None) -> np.ndarray:
    """( silu(m Wg^T) * (m Wu^T) ) Wd^T with silu(z) = z / (1 + exp(-z)).
    `store` (optional) is applied to the gated intermediate before the down projection;
    `linear` (optional) replaces y = x W^T (see decoder_layer)."""
    st = store or _keep
    lin = linear or _matmul_t
    gate = lin(m, wg)
    up = lin(m, wu)
    h = st(gate / (1.0 + np.exp(-gate)) * up)
    return lin(h, wd)


def _qkv(a, W, cfg, positions, st=_keep, lin=_matmul_t):
    N = a.shape[0]
    hd = cfg.head_dim
    q = lin(a, W["wq"])
    k = lin(a, W["wk"])
    v = lin(a, W["wv"])
    if cfg.qkv_bias:
        q = q + W["bq"]
        k = k + W["bk"]
        v = v + W["bv"]
    q = st(rope(q.reshape(N, cfg.n_q_heads, hd), positions, cfg.rope_theta))
    k = st(rope(k.reshape(N, cfg.n_kv_heads, hd), positions, cfg.rope_theta))
    v = st(v.reshape(N, cfg.n_kv_heads, hd))
    return q, k, v


def decoder_layer(x: np.ndarray, W: dict, cfg, mlp_chunk: int | None = None,
                  last_row_only: bool = False, store=None, linear=None) -> np.ndarray:
    """One pre-norm decoder block on the residual stream x [N, d].

    last_row_only: K and V are formed for every position but the query, attention
    output, O-projection and MLP only for position N-1 (enough when no later layer
    reads the other rows); returns [1, d].
    store: see the module header (None = nothing is rounded).
    linear: optional function (x [M, K], W [N, K]) -> [M, N] used for the block's seven linear
    layers in place of x W^T (the FP8-dynamic variant passes fp8_oracle.dynamic_linear)."""
    st = store or _keep
    lin = linear or _matmul_t
    N = x.shape[0]
    pos = np.arange(N)
    a = st(rmsnorm(x, W["attn_norm"], cfg.rms_eps))
    q, k, v = _qkv(a, W, cfg, pos, st, lin)
    rows = np.array([N - 1]) if last_row_only else None
    o = st(causal_gqa_attention(q, k, v, rows))
    xr = x[N - 1:N] if last_row_only else x
    xr = st(xr + lin(o.reshape(o.shape[0], -1), W["wo"]))
    m = st(rmsnorm(xr, W["mlp_norm"], cfg.rms_eps))
    if mlp_chunk is None:
        y = swiglu_mlp(m, W["wg"], W["wu"], W["wd"], store, linear)
    else:
        # Section 4.2/4.3: the position-wise part evaluated chunk by chunk over tokens,
        # each chunk written into its slice of a preallocated output.
        y = np.empty_like(xr)
        for s0 in range(0, xr.shape[0], mlp_chunk):
            y[s0:s0 + mlp_chunk] = swiglu_mlp(m[s0:s0 + mlp_chunk], W["wg"], W["wu"], W["wd"], store, linear)
    return st(xr + y)


def forward_hidden(tokens: np.ndarray, embed: np.ndarray, layers, cfg,
                   mlp_chunk: int | None = None, lazy_last_layer: bool = False, store=None, linear=None) -> np.ndarray:
    """Residual stream after all layers.  `layers` is an iterable yielding one dict of
    float64 arrays per layer (so a large model can be streamed).  Returns [N, d], or
    [1, d] (the last position) when lazy_last_layer is set."""
    tokens = np.asarray(tokens)
    x = np.asarray(embed, dtype=np.float64)[tokens]
    L = cfg.n_layers
    for l, W in enumerate(layers):
        lazy = lazy_last_layer and (l == L - 1)
        x = decoder_layer(x, W, cfg, mlp_chunk, last_row_only=lazy, store=store, linear=linear)
    return x


def last_token_logits(x_last: np.ndarray, final_norm: np.ndarray, lm_head: np.ndarray,
                      eps: float, store=None) -> np.ndarray:
    """z = rmsnorm(x_{N-1}) @ Wlm^T over the full vocabulary (`store` applies to the
    normalised row)."""
    st = store or _keep
    return st(rmsnorm(np.asarray(x_last, dtype=np.float64).reshape(-1), final_norm, eps)) @ \
        np.asarray(lm_head, dtype=np.float64).T


def candidate_logprobs(z: np.ndarray, cand: np.ndarray) -> np.ndarray:
    """Log-probabilities restricted to the acceptable-token list (Section 2.2: the
    probabilities of the acceptable tokens sum to 1): lp_i = z[c_i] - log sum_j exp z[c_j]."""
    zc = np.asarray(z, dtype=np.float64)[np.asarray(cand)]
    m = np.max(zc)
    return zc - (m + np.log(np.sum(np.exp(zc - m))))


def full_vocab_logprobs(z: np.ndarray, ids: np.ndarray) -> np.ndarray:
    """Ordinary log-softmax over the whole vocabulary, read at `ids`."""
    z = np.asarray(z, dtype=np.float64)
    m = np.max(z)
    return z[np.asarray(ids)] - (m + np.log(np.sum(np.exp(z - m))))


def prefill(tokens: np.ndarray, embed, layers, final_norm, lm_head, cfg,
            cand: np.ndarray | None = None, mlp_chunk: int | None = None,
            lazy_last_layer: bool = False, store=None, linear=None):
    """Whole path: tokens -> (last-token logits [V], candidate log-probs or None).
    `linear` replaces the decoder blocks' linear layers (never the LM head)."""
    x = forward_hidden(tokens, embed, layers, cfg, mlp_chunk, lazy_last_layer, store, linear)
    z = last_token_logits(x[-1], final_norm, lm_head, cfg.rms_eps, store)
    lp = None if cand is None else candidate_logprobs(z, cand)
    return z, lp
