"""Seeded synthetic inputs: model shapes, random-init weights, token ids, request lengths.

This module only *draws data*.  It holds none of the method's arithmetic (no norm, no
rotary embedding, no attention, no matmul), imports neither the HIP binding nor the CPU
oracle, and is the one piece both sides are fed from: the tests hand the very same
arrays to the oracle and to the library.

Recipe (random-init stand-ins for the paper's Llama-3.1-8B / Qwen-32B workloads,
Section 7 "Evaluation" model table; the trained checkpoints are not needed because the
forward pass cost and memory depend on shapes only):

* weight matrices and the embedding:  N(0, 0.02^2)
* norm gains:                         1 + N(0, 0.02^2)   (a gain of exactly 1 would hide
                                      a missing multiply, N(0,0.02) would zero the block)
* QKV biases (when enabled):          N(0, 0.02^2)
* values are rounded to the storage dtype (bf16: round-to-nearest-even) on the host,
  so both consumers see identical stored numbers
* token ids:                          uniform in [0, vocab)
* request lengths (mixed batch):      round(exp(ln(median) + sigma*z)), clipped

Every tensor has its own counter-based stream: Philox keyed by (seed, kind, layer), so
tensors can be generated in any order, layer by layer, or in parallel.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Iterator, Optional, Tuple

import numpy as np

# ----------------------------------------------------------------------------------------
# model shapes
# ----------------------------------------------------------------------------------------

F32 = 0
BF16 = 1
BF16_FP8 = 2     # bf16 model whose decoder linear layers run FP8-dynamic (weights are still given as bf16)


@dataclasses.dataclass(frozen=True)
class ModelConfig:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    vocab_size: int
    rms_eps: float
    rope_theta: float
    dtype: int = BF16          # F32, BF16 or BF16_FP8 (storage + activation dtype)
    qkv_bias: int = 0

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def replace(self, **kw) -> "ModelConfig":
        return dataclasses.replace(self, **kw)


# The five workload shapes.  "tiny" is the fp32 correctness config; the two large ones
# are Llama-3-8B-shaped and Qwen2.5-32B-shaped (shape only; random weights).
TINY = ModelConfig(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
                   ffn_dim=688, vocab_size=1024, rms_eps=1e-5, rope_theta=10000.0,
                   dtype=F32)
LLAMA8B = ModelConfig(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                      ffn_dim=14336, vocab_size=128256, rms_eps=1e-5, rope_theta=500000.0,
                      dtype=BF16)
QWEN32B = ModelConfig(n_layers=64, d_model=5120, n_q_heads=40, n_kv_heads=8, head_dim=128,
                      ffn_dim=27648, vocab_size=152064, rms_eps=1e-6, rope_theta=1000000.0,
                      dtype=BF16)


def label_ids(cfg: ModelConfig) -> np.ndarray:
    """The two fixed acceptable-token ids used everywhere: floor(V/3), floor(2V/3)."""
    return np.array([cfg.vocab_size // 3, (2 * cfg.vocab_size) // 3], dtype=np.int32)


# ----------------------------------------------------------------------------------------
# tensor kinds (the numbering is shared with include/po.h: po_tensor_kind)
# ----------------------------------------------------------------------------------------

KIND_EMBED = 0        # [V, d]
KIND_ATTN_NORM = 1    # [d]
KIND_WQ = 2           # [Hq*hd, d]     (out_features, in_features), row-major
KIND_WK = 3           # [Hkv*hd, d]
KIND_WV = 4           # [Hkv*hd, d]
KIND_BQ = 5           # [Hq*hd]
KIND_BK = 6           # [Hkv*hd]
KIND_BV = 7           # [Hkv*hd]
KIND_WO = 8           # [d, Hq*hd]
KIND_MLP_NORM = 9     # [d]
KIND_WG = 10          # [F, d]
KIND_WU = 11          # [F, d]
KIND_WD = 12          # [d, F]
KIND_FINAL_NORM = 13  # [d]
KIND_LM_HEAD = 14     # [V, d]

KIND_NAMES = {
    KIND_EMBED: "embed", KIND_ATTN_NORM: "attn_norm", KIND_WQ: "wq", KIND_WK: "wk",
    KIND_WV: "wv", KIND_BQ: "bq", KIND_BK: "bk", KIND_BV: "bv", KIND_WO: "wo",
    KIND_MLP_NORM: "mlp_norm", KIND_WG: "wg", KIND_WU: "wu", KIND_WD: "wd",
    KIND_FINAL_NORM: "final_norm", KIND_LM_HEAD: "lm_head",
}
GLOBAL_KINDS = (KIND_EMBED, KIND_FINAL_NORM, KIND_LM_HEAD)
NORM_KINDS = (KIND_ATTN_NORM, KIND_MLP_NORM, KIND_FINAL_NORM)
BIAS_KINDS = (KIND_BQ, KIND_BK, KIND_BV)


def layer_kinds(cfg: ModelConfig) -> Tuple[int, ...]:
    kinds = [KIND_ATTN_NORM, KIND_WQ, KIND_WK, KIND_WV]
    if cfg.qkv_bias:
        kinds += [KIND_BQ, KIND_BK, KIND_BV]
    kinds += [KIND_WO, KIND_MLP_NORM, KIND_WG, KIND_WU, KIND_WD]
    return tuple(kinds)


def tensor_shape(cfg: ModelConfig, kind: int) -> Tuple[int, ...]:
    d, F, V = cfg.d_model, cfg.ffn_dim, cfg.vocab_size
    return {
        KIND_EMBED: (V, d), KIND_ATTN_NORM: (d,), KIND_WQ: (cfg.q_dim, d),
        KIND_WK: (cfg.kv_dim, d), KIND_WV: (cfg.kv_dim, d), KIND_BQ: (cfg.q_dim,),
        KIND_BK: (cfg.kv_dim,), KIND_BV: (cfg.kv_dim,), KIND_WO: (d, cfg.q_dim),
        KIND_MLP_NORM: (d,), KIND_WG: (F, d), KIND_WU: (F, d), KIND_WD: (d, F),
        KIND_FINAL_NORM: (d,), KIND_LM_HEAD: (V, d),
    }[kind]


# ----------------------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions (a storage format, not arithmetic of the method)
# ----------------------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def stored_to_f64(a: np.ndarray) -> np.ndarray:
    """Stored tensor (fp32 array, or uint16 array of bf16 bits) -> exact float64 values."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# ----------------------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------------------

def _rng(seed: int, kind: int, layer: int) -> np.random.Generator:
    # Philox takes a 2x64-bit key: (seed, kind and layer packed together).
    return np.random.Generator(np.random.Philox(key=[int(seed), (int(kind) << 32) | (int(layer) + 1)]))


def make_tensor(cfg: ModelConfig, seed: int, kind: int, layer: int = -1) -> np.ndarray:
    """One stored tensor.  fp32 model -> float32 array; bf16 model -> uint16 bf16 bits."""
    shape = tensor_shape(cfg, kind)
    n = int(np.prod(shape))
    g = _rng(seed, kind, layer)
    x = g.standard_normal(n, dtype=np.float32)
    x *= np.float32(0.02)
    if kind in NORM_KINDS:
        x += np.float32(1.0)
    x = x.reshape(shape)
    if cfg.dtype != F32:
        return f32_to_bf16_bits(x)
    return x


def layer_tensors(cfg: ModelConfig, seed: int, layer: int) -> Dict[int, np.ndarray]:
    return {k: make_tensor(cfg, seed, k, layer) for k in layer_kinds(cfg)}


def global_tensors(cfg: ModelConfig, seed: int) -> Dict[int, np.ndarray]:
    return {k: make_tensor(cfg, seed, k, -1) for k in GLOBAL_KINDS}


def iter_model_tensors(cfg: ModelConfig, seed: int, threads: int = 1
                       ) -> Iterator[Tuple[int, int, np.ndarray]]:
    """Yield (kind, layer, array) for the whole model, streaming (never the whole model
    in host memory at once).  `threads` > 1 generates several tensors concurrently."""
    jobs = [(k, -1) for k in GLOBAL_KINDS]
    for l in range(cfg.n_layers):
        jobs += [(k, l) for k in layer_kinds(cfg)]
    if threads <= 1:
        for k, l in jobs:
            yield k, l, make_tensor(cfg, seed, k, l)
        return
    with ThreadPoolExecutor(max_workers=threads) as ex:
        window = 2 * threads
        pending = []
        it = iter(jobs)
        for k, l in it:
            pending.append((k, l, ex.submit(make_tensor, cfg, seed, k, l)))
            if len(pending) >= window:
                kk, ll, fut = pending.pop(0)
                yield kk, ll, fut.result()
        for kk, ll, fut in pending:
            yield kk, ll, fut.result()


def make_tokens(cfg: ModelConfig, seed: int, n: int, request: int = 0) -> np.ndarray:
    """n token ids uniform in [0, vocab)."""
    g = np.random.Generator(np.random.Philox(key=[int(seed), (1 << 48) | int(request)]))
    return g.integers(0, cfg.vocab_size, size=int(n), dtype=np.int32)


def make_lengths(seed: int, n_req: int, median: float = 2048.0, sigma: float = 0.8,
                 lo: int = 256, hi: int = 8192) -> np.ndarray:
    """Request lengths for the mixed batch: lognormal around `median`, clipped to [lo, hi]."""
    g = np.random.Generator(np.random.Philox(key=[int(seed), (2 << 48)]))
    z = g.standard_normal(int(n_req))
    lens = np.rint(np.exp(np.log(median) + sigma * z)).astype(np.int64)
    return np.clip(lens, lo, hi)


# The five workloads: (config, weight seed, token seed, length seed or None, chunk)
WORKLOADS = {
    "tiny_512": dict(cfg=TINY, wseed=1001, tseed=2001, lens=[512], chunk=512),
    "llama8b_mixed16": dict(cfg=LLAMA8B, wseed=1002, tseed=2002, lseed=3002, n_req=16, chunk=4096),
    "llama8b_32k": dict(cfg=LLAMA8B, wseed=1002, tseed=2003, lens=[32768], chunk=4096),
    "llama8b_128k": dict(cfg=LLAMA8B, wseed=1002, tseed=2004, lens=[131072], chunk=8192),
    "qwen32b_8x16k": dict(cfg=QWEN32B, wseed=1005, tseed=2005, lens=[16384] * 8, chunk=4096),
}


def workload_lengths(name: str) -> np.ndarray:
    w = WORKLOADS[name]
    if "lens" in w:
        return np.asarray(w["lens"], dtype=np.int64)
    return make_lengths(w["lseed"], w["n_req"])


# Serving traces with the structure of the paper's two evaluation workloads (Section 7.1, dataset
# table): synthetic token ids, the table's user counts, lengths and sharing pattern.
#   postrec: every user has a profile of profile_lo..profile_hi tokens and posts_per_user requests,
#            each the profile followed by one post of post_len tokens (so a user's requests share the profile);
#   credit:  every user has one request of profile_lo..profile_hi tokens, nothing shared.
SERVING = {
    "postrec": dict(n_users=20, posts_per_user=50, profile_lo=11000, profile_hi=17000, post_len=150),
    "credit": dict(n_users=60, posts_per_user=1, profile_lo=40000, profile_hi=60000, post_len=0),
}


def make_serving_trace(cfg: ModelConfig, name: str, seed: int, n_users: int = 0, posts_per_user: int = 0,
                       scale: float = 1.0):
    """-> list of (user, tokens), user by user; `scale` shrinks every length (tests), the two counts
    override the table's."""
    r = dict(SERVING[name])
    if n_users:
        r["n_users"] = n_users
    if posts_per_user:
        r["posts_per_user"] = posts_per_user
    g = np.random.Generator(np.random.Philox(key=[int(seed), (3 << 48)]))
    out = []
    for u in range(r["n_users"]):
        n_prof = max(1, int(round(int(g.integers(r["profile_lo"], r["profile_hi"] + 1)) * scale)))
        profile = make_tokens(cfg, seed, n_prof, request=1_000_000 + u)
        n_post = int(round(r["post_len"] * scale)) if r["post_len"] else 0
        for k in range(r["posts_per_user"]):
            if n_post:
                post = make_tokens(cfg, seed, n_post, request=2_000_000 + u * 10_000 + k)
                out.append((u, np.concatenate([profile, post])))
            else:
                out.append((u, profile))
    return out


def poisson_user_arrivals(seed: int, n_users: int, users_per_second: float) -> np.ndarray:
    """Arrival time of each user (all of a user's requests arrive with the user): a Poisson process."""
    g = np.random.Generator(np.random.Philox(key=[int(seed), (4 << 48)]))
    return np.cumsum(g.exponential(1.0 / users_per_second, size=int(n_users)))
