"""Shared test plumbing: turn generated tensors into what each side consumes."""
import numpy as np

from paper_2505_07203_amd import inputs as I


def oracle_layer(cfg, seed, layer):
    """One layer's weights as float64 arrays keyed by the oracle's names."""
    return {I.KIND_NAMES[k]: I.stored_to_f64(a) for k, a in I.layer_tensors(cfg, seed, layer).items()}


def oracle_layers(cfg, seed):
    """Generator over layers (streams: one layer in memory at a time)."""
    for l in range(cfg.n_layers):
        yield oracle_layer(cfg, seed, l)


def oracle_globals(cfg, seed):
    g = I.global_tensors(cfg, seed)
    return (I.stored_to_f64(g[I.KIND_EMBED]), I.stored_to_f64(g[I.KIND_FINAL_NORM]),
            I.stored_to_f64(g[I.KIND_LM_HEAD]))


def oracle_prefill(cfg, wseed, tokens, cand=None, mlp_chunk=None, lazy_last_layer=False, store=None, linear=None):
    from oracle import prefill_oracle as O
    embed, fnorm, lm = oracle_globals(cfg, wseed)
    return O.prefill(tokens, embed, oracle_layers(cfg, wseed), fnorm, lm, cfg, cand=cand,
                     mlp_chunk=mlp_chunk, lazy_last_layer=lazy_last_layer, store=store, linear=linear)


def normalised_max_rel(got, ref):
    """max_i |got_i - ref_i| / max_i |ref_i|  (relative error normalised by the oracle's
    logit range: an element-wise ratio is unbounded for logits near zero)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
