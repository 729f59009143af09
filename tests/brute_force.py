"""Scalar, loop-by-loop evaluation of the decoder forward pass on tiny inputs.

A second, deliberately different statement of the same mathematics as oracle/: Python
floats, `math` functions, explicit loops over every index, the full score row formed and
masked explicitly.  It exists only to pin oracle/prefill_oracle.py (tests/test_oracle_pins.py);
it imports neither the oracle nor the HIP binding.  Usable for N <= ~16, d <= ~32.
"""
import math
import struct


def bf16_scalar(v):
    """Nearest bfloat16 of a Python float, ties to even, by way of the float32 bit pattern
    (pure-Python counterpart of the oracle's array rounding)."""
    (u,) = struct.unpack("<I", struct.pack("<f", v))     # struct rounds to float32, ties to even
    low = u & 0xFFFF
    u >>= 16
    if low > 0x8000 or (low == 0x8000 and (u & 1)):
        u += 1
    (out,) = struct.unpack("<f", struct.pack("<I", (u << 16) & 0xFFFFFFFF))
    return out


def _dot(a, b):
    s = 0.0
    for x, y in zip(a, b):
        s += x * y
    return s


def _matvec(W, x):            # W: [out][in] nested lists
    return [_dot(row, x) for row in W]


def _rmsnorm(x, g, eps):
    ms = sum(v * v for v in x) / len(x)
    r = 1.0 / math.sqrt(ms + eps)
    return [v * r * gj for v, gj in zip(x, g)]


def _rope_vec(u, t, theta):
    hd = len(u)
    half = hd // 2
    out = [0.0] * hd
    for i in range(half):
        ang = t * theta ** (-(2.0 * i) / hd)
        c, s = math.cos(ang), math.sin(ang)
        out[i] = u[i] * c - u[i + half] * s
        out[i + half] = u[i + half] * c + u[i] * s
    return out


def forward_last_logits(tokens, embed, layers, final_norm, lm_head, cfg, store=None):
    """tokens: list[int]; embed/lm_head: nested lists [V][d]; layers: list of dicts of
    nested lists keyed like the oracle ("attn_norm","wq","wk","wv","wo","mlp_norm","wg",
    "wu","wd", optional "bq","bk","bv").  Returns (logits list [V], hidden rows [N][d]).
    `store` (optional scalar function) is applied to every element of the tensors kept
    between operators: both normalised activations, rotated Q and K, V, the attention
    output, the gated MLP intermediate and the residual stream after each update."""
    def st(vec):
        return vec if store is None else [store(e) for e in vec]
    N = len(tokens)
    hd, Hq, Hkv = cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads
    G = Hq // Hkv
    x = [list(embed[t]) for t in tokens]
    for W in layers:
        q = [[None] * Hq for _ in range(N)]
        k = [[None] * Hkv for _ in range(N)]
        v = [[None] * Hkv for _ in range(N)]
        for t in range(N):
            a = st(_rmsnorm(x[t], W["attn_norm"], cfg.rms_eps))
            qf, kf, vf = _matvec(W["wq"], a), _matvec(W["wk"], a), _matvec(W["wv"], a)
            if cfg.qkv_bias:
                qf = [p + b for p, b in zip(qf, W["bq"])]
                kf = [p + b for p, b in zip(kf, W["bk"])]
                vf = [p + b for p, b in zip(vf, W["bv"])]
            for h in range(Hq):
                q[t][h] = st(_rope_vec(qf[h * hd:(h + 1) * hd], t, cfg.rope_theta))
            for c in range(Hkv):
                k[t][c] = st(_rope_vec(kf[c * hd:(c + 1) * hd], t, cfg.rope_theta))
                v[t][c] = st(vf[c * hd:(c + 1) * hd])
        for t in range(N):
            o = []
            for h in range(Hq):
                c = h // G
                # full score row with an explicit -inf mask
                row = []
                for s in range(N):
                    row.append(_dot(q[t][h], k[s][c]) / math.sqrt(hd) if s <= t else -math.inf)
                mx = max(row)
                e = [math.exp(r - mx) for r in row]
                z = sum(e)
                oh = [0.0] * hd
                for s in range(N):
                    p = e[s] / z
                    for j in range(hd):
                        oh[j] += p * v[s][c][j]
                o += oh
            att = _matvec(W["wo"], st(o))
            x[t] = st([xi + ai for xi, ai in zip(x[t], att)])
            m = st(_rmsnorm(x[t], W["mlp_norm"], cfg.rms_eps))
            gate, up = _matvec(W["wg"], m), _matvec(W["wu"], m)
            hmid = st([gv / (1.0 + math.exp(-gv)) * uv for gv, uv in zip(gate, up)])
            y = _matvec(W["wd"], hmid)
            x[t] = st([xi + yi for xi, yi in zip(x[t], y)])
    xn = st(_rmsnorm(x[N - 1], final_norm, cfg.rms_eps))
    return _matvec(lm_head, xn), x
