"""Host-side checks that need no GPU: the library loads and exports every symbol the header
declares, the closed-form arena sizes, argument validation that happens before any launch,
and the size arithmetic the paper prints."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2505_07203_amd import binding as B
from paper_2505_07203_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "po.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(po_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = header_symbols()
    assert len(names) >= 18
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names


def test_strerror_is_distinct_per_status():
    L = B.lib()
    msgs = {L.po_strerror(s).decode() for s in range(9)}
    assert len(msgs) == 9


def expected_workspace(cfg, n, c):
    """The closed form: residual stream + Q/O + ONE layer of K/V (+ V^T copy for bf16) + one
    chunk of position-wise intermediates + rotary table + logits (each rounded up to 256 B)."""
    esz = 4 if cfg.dtype == I.F32 else 2
    al = lambda b: (b + 255) // 256 * 256
    c = min(c, n)
    parts = [n * 4, n * cfg.d_model * esz, n * cfg.q_dim * esz, n * cfg.kv_dim * esz]
    if cfg.dtype == I.BF16:       # V is kept transposed only
        parts.append(cfg.kv_dim * ((n + 63) // 64 * 64) * esz)
    else:
        parts.append(n * cfg.kv_dim * esz)
    parts += [c * cfg.d_model * esz, c * cfg.ffn_dim * esz]
    if cfg.dtype == I.F32:
        parts.append(c * 2 * cfg.ffn_dim * esz)
    parts += [n * (cfg.head_dim // 2) * 4] * 2
    parts += [cfg.vocab_size * 4, cfg.d_model * esz, 4096 * 4, 4096 * 4]
    if cfg.dtype == I.BF16:       # one word per 256-row attention tile and head (tiles to recompute with a running maximum)
        parts.append((n + 255) // 256 * cfg.n_q_heads * 4)
    parts.append(8)               # result word of the profile run's scan
    return sum(al(p) for p in parts)


@pytest.mark.parametrize("name", list(I.WORKLOADS))
def test_workspace_closed_form(name):
    w = I.WORKLOADS[name]
    cfg = w["cfg"]
    n = int(I.workload_lengths(name).max())
    wb, sb = B.po_workspace_bytes(cfg, n, w["chunk"])
    assert sb == expected_workspace(cfg, n, w["chunk"])
    esz = 4 if cfg.dtype == I.F32 else 2
    params = 2 * cfg.vocab_size * cfg.d_model + cfg.d_model + cfg.n_layers * (
        2 * cfg.d_model + (cfg.q_dim + 2 * cfg.kv_dim) * cfg.d_model + cfg.d_model * cfg.q_dim
        + 3 * cfg.ffn_dim * cfg.d_model)
    assert params * esz <= wb <= params * esz + 256 * (3 + 7 * cfg.n_layers)


def test_activation_footprint_slope_is_one_layer_of_kv():
    """Only the current layer's K/V is resident (abstract / Section 1): the per-token slope
    of the workspace must not grow with the number of layers."""
    cfg = I.LLAMA8B
    _, s1 = B.po_workspace_bytes(cfg, 65536, 4096)
    _, s2 = B.po_workspace_bytes(cfg, 131072, 4096)
    slope = (s2 - s1) / 65536
    # X + Q/O + K + V^T (bf16) + rotary table + token id + one attention word per 256 rows and head
    assert slope == 2 * (4096 + 4096 + 2 * 1024) + 2 * 4 * 64 + 4 + 32 * 4 / 256
    _, s3 = B.po_workspace_bytes(cfg.replace(n_layers=64), 131072, 4096)
    assert s3 == s2
    all_layer_kv = 2 * cfg.n_layers * cfg.kv_dim * 2
    assert slope < all_layer_kv / 5


@pytest.mark.parametrize("cfg,chunk", [(I.LLAMA8B, 4096), (I.QWEN32B, 4096), (I.TINY, 512),
                                       (I.QWEN32B.replace(dtype=I.BF16_FP8), 4096)])
def test_max_input_len_is_the_largest_length_that_fits(cfg, chunk):
    """Section 3 / the paper's maximum-input-length metric: bisection on the closed form."""
    for budget in (24e9, 40e9, 80e9, 288e9):
        budget = int(budget)
        wb1, sb1 = B.po_workspace_bytes(cfg, 1, chunk)
        if wb1 + sb1 > budget:
            with pytest.raises(B.PoError):
                B.po_max_input_len(cfg, chunk, budget)
            continue
        n = B.po_max_input_len(cfg, chunk, budget)
        wb, sb = B.po_workspace_bytes(cfg, n, chunk)
        assert wb + sb <= budget
        if n < (1 << 24):
            try:
                wb2, sb2 = B.po_workspace_bytes(cfg, n + 1, chunk)
                assert wb2 + sb2 > budget
            except B.PoError:
                pass            # n is the longest sequence the kernels address
    # the 8B shape in the 24 GB of the paper's smallest GPU: (budget - weights - chunk scratch) / slope
    if cfg is I.LLAMA8B:
        n = B.po_max_input_len(cfg, chunk, int(24e9))
        wb, _ = B.po_workspace_bytes(cfg, 1, chunk)
        assert abs(n - (24e9 - wb - 2 * 4096 * (4096 + 14336) - 4 * 128256) / 20996) < 2000
        # all-layer KV + unchunked MLP would pay 249856 bytes per token instead of 20996
        assert n > 10 * (24e9 - wb) / 249856 * 0.9


def test_paper_size_arithmetic():
    vals = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_sizes.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split(";")[0].split("=")
            vals[k.strip()] = float(v)
    cfg = I.LLAMA8B
    assert 2 * cfg.ffn_dim == vals["mlp_intermediate_numbers_per_token"]
    assert 2 * cfg.ffn_dim / (2 * cfg.kv_dim) == vals["mlp_over_one_layer_kv_ratio"]
    kv_bytes = 100000 * cfg.n_layers * 2 * cfg.kv_dim * 2
    assert abs(kv_bytes / 2 ** 30 - vals["all_layer_kv_gb_for_100000_tokens"]) < 1.5
    assert I.workload_lengths("llama8b_32k")[0] == vals["profiled_prefill_tokens"]


def test_bad_arguments_rejected_before_any_launch():
    L = B.lib()
    w, s = C.c_size_t(), C.c_size_t()
    cc = B.config_c(I.TINY)
    assert L.po_workspace_bytes(None, 512, 512, C.byref(w), C.byref(s)) == B.PO_ERR_INVALID_ARG
    assert L.po_workspace_bytes(C.byref(cc), 0, 512, C.byref(w), C.byref(s)) == B.PO_ERR_INVALID_ARG
    assert L.po_workspace_bytes(C.byref(cc), 512, 0, C.byref(w), C.byref(s)) == B.PO_ERR_INVALID_ARG
    assert L.po_workspace_bytes(C.byref(cc), 1 << 30, 512, C.byref(w), C.byref(s)) == B.PO_ERR_TOO_LONG
    bad = B.config_c(I.TINY.replace(n_kv_heads=3))
    assert L.po_workspace_bytes(C.byref(bad), 512, 512, C.byref(w), C.byref(s)) == B.PO_ERR_BAD_CONFIG
    bad = B.config_c(I.TINY.replace(dtype=7))
    assert L.po_workspace_bytes(C.byref(bad), 512, 512, C.byref(w), C.byref(s)) == B.PO_ERR_INVALID_ARG
    bad = B.config_c(I.LLAMA8B.replace(head_dim=96))
    assert L.po_workspace_bytes(C.byref(bad), 512, 512, C.byref(w), C.byref(s)) == B.PO_ERR_BAD_CONFIG
    bad = B.config_c(I.LLAMA8B.replace(ffn_dim=14336 + 8))
    assert L.po_workspace_bytes(C.byref(bad), 512, 512, C.byref(w), C.byref(s)) == B.PO_ERR_BAD_CONFIG
    # po_create: misaligned or too-small arenas are refused before any HIP call
    h = C.c_void_p()
    assert L.po_create(C.byref(cc), 512, 512, 256 + 8, 1 << 30, 4096, 1 << 30, None, C.byref(h)) == B.PO_ERR_INVALID_ARG
    assert L.po_create(C.byref(cc), 512, 512, 4096, 16, 8192, 1 << 30, None, C.byref(h)) == B.PO_ERR_WORKSPACE_TOO_SMALL
    assert L.po_create(C.byref(cc), 512, 512, None, 1 << 30, 8192, 1 << 30, None, C.byref(h)) == B.PO_ERR_INVALID_ARG
    # NULL context
    assert L.po_prefill(None, None, 1, None, 0, None, None) == B.PO_ERR_INVALID_ARG
    assert L.po_is_loaded(None) == 0
    assert L.po_get_stats(None, None) == B.PO_ERR_INVALID_ARG
    L.po_destroy(None)
    # single-kernel entry points validate too
    assert L.po_op_linear(B.PO_BF16, 4096, 4096, 4096, None, 8, 48, 64, None) == B.PO_ERR_BAD_CONFIG
    assert L.po_op_linear(3, 4096, 4096, 4096, None, 8, 64, 64, None) == B.PO_ERR_INVALID_ARG
    assert L.po_op_attention(B.PO_BF16, 4096, 4096, 4096, 4096, 4096, 8, 4, 2, 96, 0, None) == B.PO_ERR_BAD_CONFIG
    assert L.po_op_attention(B.PO_F32, 4096, 4096, 4096, 4096, None, 8, 4, 2, 64, 1, None) == B.PO_ERR_INVALID_ARG
    assert L.po_op_attention(B.PO_BF16, 4096, 4096, 4096, 4096, 4096, 8, 4, 3, 128, 0, None) == B.PO_ERR_INVALID_ARG


def test_fp8_arenas():
    """FP8-dynamic linear layers: one byte per weight of the decoder blocks' matrices plus a float32 scale per
    output channel; the workspace grows by one float32 scale per row of a launch."""
    cfg = I.LLAMA8B
    wb16, _ = B.po_workspace_bytes(cfg, 4096, 4096)
    wb8, sb8 = B.po_workspace_bytes(cfg.replace(dtype=I.BF16_FP8), 4096, 4096)
    lin = cfg.n_layers * ((cfg.q_dim + 2 * cfg.kv_dim) * cfg.d_model + cfg.d_model * cfg.q_dim + 3 * cfg.ffn_dim * cfg.d_model)
    rows = cfg.n_layers * (cfg.q_dim + 2 * cfg.kv_dim + 2 * cfg.d_model + 2 * cfg.ffn_dim)
    assert 0 <= wb8 - (wb16 - lin + 4 * rows) <= 256 * 4 * cfg.n_layers
    _, sb16 = B.po_workspace_bytes(cfg, 4096, 4096)
    assert sb8 - sb16 == 4 * 4096 * cfg.ffn_dim // cfg.d_model
    # shapes the FP8 kernels cannot take are refused up front
    with pytest.raises(B.PoError):
        B.po_workspace_bytes(I.TINY.replace(dtype=I.BF16_FP8, ffn_dim=704), 512, 128)      # 704 is not a multiple of 128


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N > 1 exits with a message instead of measuring something else."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_serving_traces_have_the_papers_structure():
    """Section 7.1 dataset table: users x posts, profile and post lengths, what is shared."""
    cfg = I.TINY
    post = I.make_serving_trace(cfg, "postrec", 5)
    assert len(post) == 20 * 50
    by_user = {}
    for u, t in post:
        by_user.setdefault(u, []).append(t)
    assert len(by_user) == 20 and all(len(v) == 50 for v in by_user.values())
    for v in by_user.values():
        n_prof = len(v[0]) - 150
        assert 11000 <= n_prof <= 17000
        assert all(len(t) == n_prof + 150 and np.array_equal(t[:n_prof], v[0][:n_prof]) for t in v)   # shared profile
        assert not np.array_equal(v[0][n_prof:], v[1][n_prof:])                                       # own post
    a, b = by_user[0][0], by_user[1][0]
    assert not np.array_equal(a[:1000], b[:1000])                                                     # nothing shared across users
    credit = I.make_serving_trace(cfg, "credit", 5)
    assert len(credit) == 60 and all(40000 <= len(t) <= 60000 for _, t in credit)
    assert all(0 <= t.min() and t.max() < cfg.vocab_size for _, t in credit[:3])
    small = I.make_serving_trace(cfg, "postrec", 5, n_users=3, posts_per_user=2, scale=0.01)
    assert len(small) == 6 and all(110 + 2 <= len(t) <= 170 + 2 for _, t in small)
    arr = I.poisson_user_arrivals(9, 1000, 4.0)
    assert np.all(np.diff(arr) > 0) and abs(arr[-1] / 1000 - 0.25) < 0.03                             # mean gap 1 / rate


def test_public_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: include/po.h must compile as C99 (and as C++) with nothing but the standard headers."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "hdr.c"
    src.write_text('#include "po.h"\nint main(void) { return (int)sizeof(po_stats) == 0; }\n')
    for cc, std in (("gcc", ["-std=c99", "-pedantic"]), ("g++", ["-std=c++17", "-x", "c++"])):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} not installed")
        r = subprocess.run([cc, *std, "-Wall", "-Werror", "-I", os.path.join(root, "include"), "-fsyntax-only", str(src)],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
