"""ctypes binding over libpo.so: the same names as include/po.h, argument marshalling only.

PyTorch appears here solely as the provider of device memory (the two arenas) and of the
HIP stream handle; every step of the path runs inside libpo's own kernels.  If libpo.so is
missing, loading fails with an error: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpo.so")

PO_OK = 0
PO_ERR_INVALID_ARG = 1
PO_ERR_BAD_CONFIG = 2
PO_ERR_NOT_LOADED = 3
PO_ERR_TOO_LONG = 4
PO_ERR_TOKEN_RANGE = 5
PO_ERR_WORKSPACE_TOO_SMALL = 6
PO_ERR_OOM = 7
PO_ERR_DEVICE = 8

PO_F32, PO_BF16, PO_BF16_FP8 = 0, 1, 2
PO_KEEP_ALL = -1
KERNEL_CLASSES = ("attention", "qkv", "residual", "gate_up")   # po_kernel_class order

EXPORTS = [
    "po_workspace_bytes", "po_create", "po_load_tensor", "po_load_weights", "po_is_loaded", "po_prefill",
    "po_prefill_batch", "po_set_phase_timing", "po_get_stats", "po_destroy", "po_strerror",
    "po_last_device_error", "po_op_rmsnorm", "po_op_linear", "po_op_gate_up_silu",
    "po_op_pack_gate_up", "po_op_attention", "po_op_rope", "po_op_lm_head", "po_op_rope_table",
    "po_op_pack_qkv", "po_op_qkv_rope", "po_max_input_len", "po_profile", "po_set_lazy_last_layer",
    "po_kv_cache_bytes", "po_attach_kv_cache", "po_prefill_prefix", "po_prefill_packed",
    "po_op_quantize_rows", "po_op_rmsnorm_quantize", "po_op_linear_fp8", "po_op_qkv_rope_fp8",
    "po_attach_kv_cache_slots", "po_kv_cache_match", "po_kv_cache_slot", "po_sched_pick_multi",
    "po_profile_jct", "po_engine_step", "po_set_few_rows_split", "po_set_storage_rounding", "po_op_linear_split", "po_sched_push_request", "po_op_attention_split",
    "po_sched_create", "po_sched_destroy", "po_sched_set_jct_model", "po_sched_fit_jct_model", "po_sched_push",
    "po_sched_size", "po_sched_pick", "po_sched_remove", "po_op_rope_static", "po_op_mfma_peak", "po_op_stream_copy",
]


class ModelConfigC(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn_dim", C.c_int32),
                ("vocab_size", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("dtype", C.c_int32), ("qkv_bias", C.c_int32)]


class StatsC(C.Structure):
    _fields_ = [("last_prefill_ms", C.c_double), ("kernel_ms", C.c_double * 4),
                ("kernel_launches", C.c_int64 * 4), ("weights_bytes", C.c_uint64),
                ("workspace_bytes", C.c_uint64), ("last_len", C.c_int64),
                ("split_launches", C.c_int64)]


class PoError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(what)


_lib = None


def lib() -> C.CDLL:
    """Loads libpo.so (built in-tree by paper_2505_07203_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it first (python -m paper_2505_07203_amd.build); "
            "there is no fallback implementation")
    # The arenas and the stream come from PyTorch, so libpo must bind to the SAME HIP runtime
    # PyTorch uses (its wheel ships its own libamdhip64 with the same soname): importing torch
    # first makes the loader resolve libpo's dependency to that already-loaded copy.  Loading
    # libpo first would pull in a second, unrelated runtime that knows none of torch's pointers.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float
    L.po_workspace_bytes.argtypes = [C.POINTER(ModelConfigC), i64, i32, C.POINTER(sz), C.POINTER(sz)]
    L.po_max_input_len.argtypes = [C.POINTER(ModelConfigC), i32, sz, C.POINTER(i64)]
    L.po_profile.argtypes = [vp, i64, C.POINTER(C.c_double), C.POINTER(sz)]
    L.po_create.argtypes = [C.POINTER(ModelConfigC), i64, i32, vp, sz, vp, sz, vp, C.POINTER(vp)]
    L.po_load_tensor.argtypes = [vp, i32, i32, vp, sz]
    L.po_load_weights.argtypes = [vp, vp]
    L.po_is_loaded.argtypes = [vp]
    L.po_prefill.argtypes = [vp, vp, i64, vp, i32, vp, vp]
    L.po_prefill_batch.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp]
    L.po_prefill_packed.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp]
    L.po_set_phase_timing.argtypes = [vp, i32]
    L.po_set_lazy_last_layer.argtypes = [vp, i32]
    L.po_kv_cache_bytes.argtypes = [C.POINTER(ModelConfigC), i64, C.POINTER(sz)]
    L.po_attach_kv_cache.argtypes = [vp, vp, sz, i64]
    L.po_attach_kv_cache_slots.argtypes = [vp, vp, sz, i64, i32]
    L.po_kv_cache_match.argtypes = [vp, vp, i64, C.POINTER(i64)]
    L.po_kv_cache_slot.argtypes = [vp, i32, vp, i64, C.POINTER(i64)]
    L.po_set_few_rows_split.argtypes = [vp, i32]
    L.po_set_storage_rounding.argtypes = [vp, i32]
    L.po_engine_step.argtypes = [vp, vp, C.c_double, vp, i32, vp, vp, i32, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64),
                                 C.POINTER(i32)]
    L.po_sched_push_request.argtypes = [vp, i64, vp, i64, vp, i32, C.c_double]
    L.po_profile_jct.argtypes = [vp, i64, i64, vp, vp, vp, i32, C.POINTER(i32)]
    L.po_sched_pick_multi.argtypes = [vp, vp, vp, i32, C.c_double, C.POINTER(i64), C.POINTER(i64)]
    L.po_prefill_prefix.argtypes = [vp, vp, i64, i64, vp, i32, vp, vp, C.POINTER(i64)]
    L.po_get_stats.argtypes = [vp, C.POINTER(StatsC)]
    L.po_destroy.argtypes = [vp]
    L.po_destroy.restype = None
    L.po_strerror.argtypes = [i32]
    L.po_strerror.restype = C.c_char_p
    L.po_last_device_error.argtypes = []
    L.po_last_device_error.restype = C.c_char_p
    L.po_op_rmsnorm.argtypes = [i32, vp, vp, vp, i64, i32, f32, vp]
    L.po_op_linear.argtypes = [i32, vp, vp, vp, vp, i64, i32, i32, vp]
    L.po_op_attention_split.argtypes = [vp, vp, vp, vp, vp, vp, sz, i64, i32, i32, i32, i64, vp, C.POINTER(i32)]
    L.po_op_linear_split.argtypes = [vp, vp, vp, vp, vp, sz, i64, i32, i32, vp, C.POINTER(i32)]
    L.po_op_gate_up_silu.argtypes = [i32, vp, vp, vp, vp, i64, i32, i32, vp]
    L.po_op_pack_gate_up.argtypes = [i32, vp, vp, vp, i32, i32, vp]
    L.po_op_attention.argtypes = [i32, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp]
    L.po_op_rope.argtypes = [i32, vp, i64, i32, i32, f32, vp]
    L.po_op_rope_static.argtypes = [i32, vp, i64, i32, i32, f32, vp]
    L.po_op_mfma_peak.argtypes = [i32, i32, i32, vp, sz, vp, vp, C.POINTER(C.c_double)]
    L.po_op_stream_copy.argtypes = [vp, vp, sz, vp]
    L.po_op_lm_head.argtypes = [i32, vp, vp, vp, i32, i32, vp]
    L.po_op_rope_table.argtypes = [vp, vp, i64, i32, f32, vp]
    L.po_op_pack_qkv.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]
    L.po_op_qkv_rope.argtypes = [vp, vp, vp, vp, vp, vp, i64, vp, vp, i64, i64, i32, i32, i32, i32, f32, vp]
    L.po_op_quantize_rows.argtypes = [vp, vp, vp, i64, i32, vp]
    L.po_op_rmsnorm_quantize.argtypes = [vp, vp, vp, vp, i64, i32, f32, vp]
    L.po_op_linear_fp8.argtypes = [i32, vp, vp, vp, vp, vp, vp, i64, i32, i32, vp]
    L.po_op_qkv_rope_fp8.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, vp, i64, i64, i32, i32, i32, i32, f32, vp]
    f64 = C.c_double
    L.po_sched_create.argtypes = [f64, C.POINTER(vp)]
    L.po_sched_destroy.argtypes = [vp]
    L.po_sched_destroy.restype = None
    L.po_sched_set_jct_model.argtypes = [vp, f64, f64, f64]
    L.po_sched_fit_jct_model.argtypes = [vp, vp, vp, vp, i32, C.POINTER(f64 * 3)]
    L.po_sched_push.argtypes = [vp, i64, vp, i64, f64]
    L.po_sched_size.argtypes = [vp]
    L.po_sched_remove.argtypes = [vp, i64]
    L.po_sched_size.restype = i64
    L.po_sched_pick.argtypes = [vp, vp, i64, f64, C.POINTER(i64), C.POINTER(i64)]
    for name in EXPORTS:
        if name not in ("po_destroy", "po_strerror", "po_last_device_error", "po_sched_destroy", "po_sched_size"):
            getattr(L, name).restype = i32
    _lib = L
    return L


def check(status: int) -> None:
    if status != PO_OK:
        L = lib()
        msg = L.po_strerror(status).decode()
        if status == PO_ERR_DEVICE:
            msg += ": " + L.po_last_device_error().decode()
        raise PoError(status, f"libpo: {msg} (status {status})")


def config_c(cfg) -> ModelConfigC:
    return ModelConfigC(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                        cfg.ffn_dim, cfg.vocab_size, cfg.rms_eps, cfg.rope_theta, cfg.dtype,
                        cfg.qkv_bias)


def po_workspace_bytes(cfg, max_input_len: int, mlp_chunk: int):
    """-> (weights_bytes, workspace_bytes); closed form, needs no GPU."""
    w, s = C.c_size_t(0), C.c_size_t(0)
    cc = config_c(cfg)
    check(lib().po_workspace_bytes(C.byref(cc), max_input_len, mlp_chunk, C.byref(w), C.byref(s)))
    return w.value, s.value


def po_max_input_len(cfg, mlp_chunk: int, hbm_budget_bytes: int) -> int:
    """Largest maximum input length whose arenas fit the budget; closed form, needs no GPU."""
    n = C.c_int64(0)
    cc = config_c(cfg)
    check(lib().po_max_input_len(C.byref(cc), mlp_chunk, hbm_budget_bytes, C.byref(n)))
    return n.value


def _host_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Context:
    """A po_ctx over two torch-allocated device arenas on the current stream."""

    def __init__(self, cfg, max_input_len: int, mlp_chunk: int, device: str = "cuda:0"):
        import torch
        self.cfg = cfg
        self.max_input_len = int(max_input_len)
        self.mlp_chunk = int(mlp_chunk)
        wb, sb = po_workspace_bytes(cfg, max_input_len, mlp_chunk)
        self.weights_bytes, self.workspace_bytes = wb, sb
        self._torch = torch
        self.device = torch.device(device)
        # plumbing only: raw byte arenas and the stream handle
        self._w = torch.empty(wb, dtype=torch.uint8, device=self.device)
        self._ws = torch.empty(sb, dtype=torch.uint8, device=self.device)
        with torch.cuda.device(self.device):
            self.stream = torch.cuda.current_stream().cuda_stream
        h = C.c_void_p()
        cc = config_c(cfg)
        check(lib().po_create(C.byref(cc), self.max_input_len, self.mlp_chunk, self._w.data_ptr(), wb,
                              self._ws.data_ptr(), sb, self.stream, C.byref(h)))
        self._h = h

    # -- same names as the C ABI ---------------------------------------------------------
    def po_load_tensor(self, kind: int, layer: int, host: np.ndarray) -> None:
        a = np.ascontiguousarray(host)
        check(lib().po_load_tensor(self._h, kind, layer, _host_ptr(a), a.nbytes))

    def po_load_weights(self, tensors) -> None:
        """tensors: {kind: array} for the global kinds, {kind: [array per layer]} for the per-layer kinds"""
        keep = []
        slots = (C.c_void_p * 15)()
        for kind, t in tensors.items():
            if isinstance(t, (list, tuple)):
                arrs = [np.ascontiguousarray(a) for a in t]
                ptrs = (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])
                keep += arrs + [ptrs]
                slots[kind] = C.cast(ptrs, C.c_void_p)
            else:
                a = np.ascontiguousarray(t)
                keep.append(a)
                slots[kind] = a.ctypes.data
        check(lib().po_load_weights(self._h, C.byref(slots)))

    def po_is_loaded(self) -> bool:
        return bool(lib().po_is_loaded(self._h))

    def po_prefill(self, tokens: np.ndarray, cand: Optional[Sequence[int]] = None,
                   want_logits: bool = True):
        """-> (logits float32[V] or None, candidate log-probs float32[n_cand] or None)"""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        n_cand = 0 if cand is None else len(cand)
        cand_a = None if cand is None else np.ascontiguousarray(cand, dtype=np.int32)
        logits = np.empty(self.cfg.vocab_size, dtype=np.float32) if want_logits else None
        lp = np.empty(n_cand, dtype=np.float32) if n_cand else None
        check(lib().po_prefill(self._h, _host_ptr(tok), tok.shape[0], _host_ptr(cand_a), n_cand,
                               _host_ptr(logits), _host_ptr(lp)))
        return logits, lp

    def po_prefill_batch(self, token_lists: Sequence[np.ndarray], cand: Optional[Sequence[int]] = None,
                         want_logits: bool = False, packed: bool = False):
        lens = np.array([len(t) for t in token_lists], dtype=np.int64)
        tok = np.ascontiguousarray(np.concatenate([np.asarray(t, dtype=np.int32) for t in token_lists]))
        n_req = len(token_lists)
        n_cand = 0 if cand is None else len(cand)
        cand_a = None if cand is None else np.ascontiguousarray(cand, dtype=np.int32)
        logits = np.empty((n_req, self.cfg.vocab_size), dtype=np.float32) if want_logits else None
        lp = np.empty((n_req, n_cand), dtype=np.float32) if n_cand else None
        entry = lib().po_prefill_packed if packed else lib().po_prefill_batch
        check(entry(self._h, _host_ptr(tok), _host_ptr(lens), n_req, _host_ptr(cand_a), n_cand, _host_ptr(logits),
                    _host_ptr(lp)))
        return logits, lp

    def po_prefill_packed(self, token_lists: Sequence[np.ndarray], cand: Optional[Sequence[int]] = None,
                          want_logits: bool = False):
        return self.po_prefill_batch(token_lists, cand, want_logits, packed=True)

    def po_profile(self, length: int):
        """-> (device ms of a fake request of `length` tokens, measured high-water mark of the arena)"""
        ms, touched = C.c_double(0), C.c_size_t(0)
        check(lib().po_profile(self._h, length, C.byref(ms), C.byref(touched)))
        return ms.value, touched.value

    def po_attach_kv_cache(self, prefix_capacity: int, n_slots: int = 1) -> int:
        """Allocates (torch) and attaches a prefix K/V cache of n_slots entries; returns its size in bytes."""
        n = C.c_size_t(0)
        cc = config_c(self.cfg)
        check(lib().po_kv_cache_bytes(C.byref(cc), prefix_capacity, C.byref(n)))
        total = n.value * n_slots
        self._kvc = self._torch.empty(total, dtype=self._torch.uint8, device=self.device)
        check(lib().po_attach_kv_cache_slots(self._h, self._kvc.data_ptr(), total, prefix_capacity, n_slots))
        self._kv_slots = n_slots
        return total

    def po_detach_kv_cache(self) -> None:
        """po_attach_kv_cache with a NULL cache: detaches and releases it."""
        check(lib().po_attach_kv_cache(self._h, None, 0, 0))
        self._kvc = None

    def po_profile_jct(self, max_len: int, step: int):
        """-> (n_input int64[], n_cached int64[], jct_ms float64[]) over the profiling grid."""
        n = C.c_int32(0)
        check(lib().po_profile_jct(self._h, max_len, step, None, None, None, 0, C.byref(n)))
        a, b = np.empty(n.value, dtype=np.int64), np.empty(n.value, dtype=np.int64)
        t = np.empty(n.value, dtype=np.float64)
        check(lib().po_profile_jct(self._h, max_len, step, _host_ptr(a), _host_ptr(b), _host_ptr(t), n.value, C.byref(n)))
        return a, b, t

    def po_kv_cache_match(self, tokens: np.ndarray) -> int:
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        out = C.c_int64(0)
        check(lib().po_kv_cache_match(self._h, _host_ptr(tok), len(tok), C.byref(out)))
        return out.value

    def po_kv_cache_slot(self, slot: int) -> np.ndarray:
        n = C.c_int64(0)
        check(lib().po_kv_cache_slot(self._h, slot, None, 0, C.byref(n)))
        out = np.empty(n.value, dtype=np.int32)
        check(lib().po_kv_cache_slot(self._h, slot, _host_ptr(out), n.value, C.byref(n)))
        return out

    def po_prefill_prefix(self, tokens: np.ndarray, keep_prefix: int, cand: Optional[Sequence[int]] = None,
                          want_logits: bool = True):
        """-> (logits or None, candidate log-probs or None, reused prefix length)"""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        n_cand = 0 if cand is None else len(cand)
        cand_a = None if cand is None else np.ascontiguousarray(cand, dtype=np.int32)
        logits = np.empty(self.cfg.vocab_size, dtype=np.float32) if want_logits else None
        lp = np.empty(n_cand, dtype=np.float32) if n_cand else None
        reused = C.c_int64(0)
        check(lib().po_prefill_prefix(self._h, _host_ptr(tok), tok.shape[0], keep_prefix, _host_ptr(cand_a), n_cand,
                                      _host_ptr(logits), _host_ptr(lp), C.byref(reused)))
        return logits, lp, reused.value

    def po_engine_step(self, sched: "Scheduler", now: float, cand: Optional[Sequence[int]] = None,
                       want_logits: bool = False, cand_capacity: int = 64):
        """-> (id or -1, length, reused prefix length, logits or None, candidate log-probs or None).
        cand=None: the list each request was pushed with (at most cand_capacity ids)."""
        n_cand = 0 if cand is None else len(cand)
        cand_a = None if cand is None else np.ascontiguousarray(cand, dtype=np.int32)
        cap = max(n_cand, cand_capacity)
        logits = np.empty(self.cfg.vocab_size, dtype=np.float32) if want_logits else None
        lp = np.empty(cap, dtype=np.float32)
        rid, n, reused, used = C.c_int64(-1), C.c_int64(0), C.c_int64(0), C.c_int32(0)
        check(lib().po_engine_step(self._h, sched._h, now, _host_ptr(cand_a), n_cand, _host_ptr(logits), _host_ptr(lp), cap,
                                   C.byref(rid), C.byref(n), C.byref(reused), C.byref(used)))
        return rid.value, n.value, reused.value, logits, (lp[:used.value] if used.value else None)

    def po_set_few_rows_split(self, on: bool) -> None:
        check(lib().po_set_few_rows_split(self._h, 1 if on else 0))

    def po_set_storage_rounding(self, on: bool) -> None:
        check(lib().po_set_storage_rounding(self._h, 1 if on else 0))

    def po_set_lazy_last_layer(self, on: bool) -> None:
        check(lib().po_set_lazy_last_layer(self._h, 1 if on else 0))

    def po_set_phase_timing(self, on: bool) -> None:
        check(lib().po_set_phase_timing(self._h, 1 if on else 0))

    def po_get_stats(self) -> dict:
        s = StatsC()
        check(lib().po_get_stats(self._h, C.byref(s)))
        out = {n: getattr(s, n) for n, _ in StatsC._fields_}
        out["kernel_ms"] = dict(zip(KERNEL_CLASSES, s.kernel_ms))
        out["kernel_launches"] = dict(zip(KERNEL_CLASSES, s.kernel_launches))
        return out

    def po_destroy(self) -> None:
        if getattr(self, "_h", None):
            lib().po_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.po_destroy()
        except Exception:
            pass

    # -- convenience: load a whole synthetic model from the seeded generator ----------------
    def load_synthetic(self, seed: int, threads: int = 8, values_of=None) -> None:
        """Seeded random-init weights of this context's configuration.  values_of=inputs.BF16 on a float32 context
        loads the bf16 model's weight VALUES (generated and rounded as for the bf16 model, handed over as float32):
        the same model evaluated in float32."""
        from . import inputs as I
        gen_cfg = self.cfg if values_of is None else self.cfg.replace(dtype=values_of)
        for kind, layer, arr in I.iter_model_tensors(gen_cfg, seed, threads=threads):
            if values_of is not None and self.cfg.dtype == I.F32 and arr.dtype == np.uint16:
                arr = I.bf16_bits_to_f32(arr)
            self.po_load_tensor(kind, layer, arr)
        if not self.po_is_loaded():
            raise RuntimeError("model not fully loaded")


def load_synthetic_models(contexts, seed: int, threads: int = 8, values_of=None) -> None:
    """Context.load_synthetic for several contexts of ONE model shape at once (say a bf16 context and a float32
    context that evaluates the same weight values): every tensor is generated once and handed to each context, which
    halves the host time of tests that compare two evaluation paths."""
    from . import inputs as I
    ref = contexts[0].cfg
    gen_cfg = ref if values_of is None else ref.replace(dtype=values_of)
    for kind, layer, arr in I.iter_model_tensors(gen_cfg, seed, threads=threads):
        for c in contexts:
            a = arr
            if c.cfg.dtype == I.F32 and arr.dtype == np.uint16:
                a = I.bf16_bits_to_f32(arr)
            c.po_load_tensor(kind, layer, a)
    for c in contexts:
        if not c.po_is_loaded():
            raise RuntimeError("model not fully loaded")


# ---- single-kernel entry points on torch device tensors (pointers only) ---------------------

def _dt(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return PO_F32
    if t.dtype == torch.bfloat16:
        return PO_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def po_op_rmsnorm(x, g, eps: float):
    import torch
    y = torch.empty_like(x)
    check(lib().po_op_rmsnorm(_dt(x), x.data_ptr(), g.data_ptr(), y.data_ptr(), x.shape[0], x.shape[1], eps, _stream()))
    return y


def po_op_linear(a, w, residual=None, out=None):
    import torch
    M, K = a.shape
    N = w.shape[0]
    c = out if out is not None else torch.empty((M, N), dtype=a.dtype, device=a.device)
    check(lib().po_op_linear(_dt(a), a.data_ptr(), w.data_ptr(), c.data_ptr(),
                             None if residual is None else residual.data_ptr(), M, N, K, _stream()))
    return c


def po_op_linear_split(a, w, residual, scratch_bytes=1 << 28):
    """-> (C or None, splits): the split-K form of po_op_linear with a residual; None when nothing was split"""
    import torch
    M, K = a.shape
    N = w.shape[0]
    c = torch.empty((M, N), dtype=a.dtype, device=a.device)
    scratch = torch.empty(scratch_bytes, dtype=torch.uint8, device=a.device)
    n = C.c_int32(0)
    check(lib().po_op_linear_split(a.data_ptr(), w.data_ptr(), c.data_ptr(), residual.data_ptr(), scratch.data_ptr(),
                                   scratch_bytes, M, N, K, _stream(), C.byref(n)))
    torch.cuda.synchronize()
    return (c if n.value > 1 else None), n.value


def po_op_quantize_rows(x, in_place=False):
    """bf16 [M, K] -> (uint8 codes [M, K], float32 scales [M]); in_place: the codes overwrite x's memory
    (returned as a uint8 view [M, 2K] whose first K columns are the codes)"""
    import torch
    M, K = x.shape
    scales = torch.empty(M, dtype=torch.float32, device=x.device)
    if in_place:
        codes = x.view(torch.uint8)
        check(lib().po_op_quantize_rows(x.data_ptr(), x.data_ptr(), scales.data_ptr(), M, K, _stream()))
        # (the library writes each row's codes at the row's own start: pitch 2K bytes)
        return codes, scales
    codes = torch.empty((M, K), dtype=torch.uint8, device=x.device)
    check(lib().po_op_quantize_rows(x.data_ptr(), codes.data_ptr(), scales.data_ptr(), M, K, _stream()))
    return codes, scales


def po_op_rmsnorm_quantize(x, g, eps):
    import torch
    M, d = x.shape
    codes = torch.empty((M, d), dtype=torch.uint8, device=x.device)
    scales = torch.empty(M, dtype=torch.float32, device=x.device)
    check(lib().po_op_rmsnorm_quantize(x.data_ptr(), g.data_ptr(), codes.data_ptr(), scales.data_ptr(), M, d, eps,
                                       _stream()))
    return codes, scales


def po_op_linear_fp8(a_codes, a_scales, w_codes, w_scales, residual=None, out=None, silu_mul=False):
    import torch
    M, K = a_codes.shape
    N = w_codes.shape[0]
    epi = 2 if silu_mul else (1 if residual is not None else 0)
    c = out if out is not None else torch.empty((M, N // 2 if silu_mul else N), dtype=torch.bfloat16, device=a_codes.device)
    check(lib().po_op_linear_fp8(epi, a_codes.data_ptr(), a_scales.data_ptr(), w_codes.data_ptr(), w_scales.data_ptr(),
                                 c.data_ptr(), None if residual is None else residual.data_ptr(), M, N, K, _stream()))
    return c


def attention_q_scale(head_dim: int) -> float:
    """log2(e) / sqrt(head_dim) as the float32 the library uses: the factor between the rotated queries and what
    po_op_attention expects with q_prescaled"""
    import math
    return float(np.float32(1.4426950408889634 / math.sqrt(head_dim)))


def po_op_qkv_rope_fp8(a_codes, a_scales, w_codes, w_scales, bqkv, cos, sin, n_q_heads, n_kv_heads, head_dim, pos0=0,
                       q_scale: float = 1.0):
    import torch
    M, K = a_codes.shape
    qd, kvd = n_q_heads * head_dim, n_kv_heads * head_dim
    ldv = (pos0 + M + 63) // 64 * 64
    q = torch.empty((M, qd), dtype=torch.bfloat16, device=a_codes.device)
    k = torch.empty((M, kvd), dtype=torch.bfloat16, device=a_codes.device)
    vt = torch.zeros((kvd, ldv), dtype=torch.bfloat16, device=a_codes.device)
    check(lib().po_op_qkv_rope_fp8(a_codes.data_ptr(), a_scales.data_ptr(), w_codes.data_ptr(), w_scales.data_ptr(),
                                   None if bqkv is None else bqkv.data_ptr(), q.data_ptr(), k.data_ptr(), vt.data_ptr(),
                                   ldv, cos.data_ptr(), sin.data_ptr(), pos0, M, n_q_heads, n_kv_heads, head_dim, K,
                                   q_scale, _stream()))
    return q, k, vt


def po_op_pack_gate_up(wg, wu):
    import torch
    F, K = wg.shape
    out = torch.empty((2 * F, K), dtype=wg.dtype, device=wg.device)
    check(lib().po_op_pack_gate_up(_dt(wg), wg.data_ptr(), wu.data_ptr(), out.data_ptr(), F, K, _stream()))
    return out


def po_op_gate_up_silu(a, wgu):
    import torch
    M, K = a.shape
    F = wgu.shape[0] // 2
    h = torch.empty((M, F), dtype=a.dtype, device=a.device)
    scratch = torch.empty((M, 2 * F), dtype=a.dtype, device=a.device) if a.dtype == torch.float32 else None
    check(lib().po_op_gate_up_silu(_dt(a), a.data_ptr(), wgu.data_ptr(), h.data_ptr(),
                                   None if scratch is None else scratch.data_ptr(), M, F, K, _stream()))
    return h


def po_op_attention(q, k, v, out=None, q_prescaled: bool = False):
    """q [N,Hq,hd], k/v [N,Hkv,hd] (rotated) -> o [N,Hq,hd]; out may be q itself.  q_prescaled: q holds the queries
    times attention_q_scale(hd)."""
    import torch
    N, Hq, hd = q.shape
    Hkv = k.shape[1]
    o = out if out is not None else torch.empty_like(q)
    scratch = None
    if q.dtype == torch.bfloat16:
        vt_bytes = (2 * Hkv * hd * ((N + 63) // 64 * 64) + 255) // 256 * 256
        scratch = torch.empty(vt_bytes + 4 * Hq * ((N + 255) // 256), dtype=torch.uint8, device=q.device)
    check(lib().po_op_attention(_dt(q), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                None if scratch is None else scratch.data_ptr(), N, Hq, Hkv, hd, 1 if q_prescaled else 0,
                                _stream()))
    return o


def po_op_attention_split(q, k, v, q_row0: int, part_bytes: int = 1 << 28):
    """-> (o or None, splits): rows [q_row0, N) by the split-key kernel; None when nothing was split"""
    import torch
    N, Hq, hd = q.shape
    Hkv = k.shape[1]
    o = torch.zeros_like(q)
    vt = torch.empty(Hkv * hd * ((N + 63) // 64 * 64), dtype=q.dtype, device=q.device)
    part = torch.empty(part_bytes, dtype=torch.uint8, device=q.device)
    n = C.c_int32(0)
    check(lib().po_op_attention_split(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), vt.data_ptr(), part.data_ptr(),
                                      part_bytes, N, Hq, Hkv, hd, q_row0, _stream(), C.byref(n)))
    torch.cuda.synchronize()
    return (o if n.value > 1 else None), n.value


def po_op_rope(x, theta: float):
    """in place on x [N, H, hd]"""
    N, H, hd = x.shape
    check(lib().po_op_rope(_dt(x), x.data_ptr(), N, H, hd, theta, _stream()))
    return x


def po_op_rope_static(x, theta: float):
    """in place on x [N, H, hd]; the variant that allocates nothing (asynchronous on the current stream)"""
    N, H, hd = x.shape
    check(lib().po_op_rope_static(_dt(x), x.data_ptr(), N, H, hd, theta, _stream()))
    return x


def po_op_mfma_peak(kind: int, waves_per_simd: int, iters: int, operands, sink) -> float:
    """launches the matrix-instruction loop on the current stream -> flop executed"""
    f = C.c_double(0)
    check(lib().po_op_mfma_peak(kind, waves_per_simd, iters, operands.data_ptr(), operands.numel() * operands.element_size(),
                                sink.data_ptr(), _stream(), C.byref(f)))
    return f.value


def po_op_stream_copy(src, dst) -> None:
    check(lib().po_op_stream_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream()))


def po_op_lm_head(x, w):
    import torch
    V, d = w.shape
    z = torch.empty(V, dtype=torch.float32, device=w.device)
    check(lib().po_op_lm_head(_dt(x), x.data_ptr(), w.data_ptr(), z.data_ptr(), V, d, _stream()))
    return z


def po_op_rope_table(n: int, head_dim: int, theta: float):
    import torch
    cos = torch.empty((n, head_dim // 2), dtype=torch.float32, device="cuda")
    sin = torch.empty_like(cos)
    check(lib().po_op_rope_table(cos.data_ptr(), sin.data_ptr(), n, head_dim, theta, _stream()))
    return cos, sin


def po_op_pack_qkv(wq, wk, wv, n_q_heads: int, n_kv_heads: int, head_dim: int, bq=None, bk=None, bv=None):
    import torch
    K = wq.shape[1]
    rows = (n_q_heads + 2 * n_kv_heads) * head_dim
    wqkv = torch.empty((rows, K), dtype=wq.dtype, device=wq.device)
    bqkv = torch.empty(rows, dtype=wq.dtype, device=wq.device) if bq is not None else None
    p = lambda t: None if t is None else t.data_ptr()
    check(lib().po_op_pack_qkv(wq.data_ptr(), wk.data_ptr(), wv.data_ptr(), wqkv.data_ptr(), p(bq), p(bk), p(bv),
                               p(bqkv), n_q_heads, n_kv_heads, head_dim, K, _stream()))
    return wqkv, bqkv


def po_op_qkv_rope(a, wqkv, bqkv, cos, sin, n_q_heads: int, n_kv_heads: int, head_dim: int, pos0: int = 0,
                   vt=None, q_scale: float = 1.0):
    """-> q [M, Hq*hd], k [M, Hkv*hd] (rotated), vt [Hkv*hd, ldv] with columns pos0..pos0+M-1 written"""
    import torch
    M, K = a.shape
    q = torch.empty((M, n_q_heads * head_dim), dtype=a.dtype, device=a.device)
    k = torch.empty((M, n_kv_heads * head_dim), dtype=a.dtype, device=a.device)
    if vt is None:
        vt = torch.zeros((n_kv_heads * head_dim, (pos0 + M + 63) // 64 * 64), dtype=a.dtype, device=a.device)
    check(lib().po_op_qkv_rope(a.data_ptr(), wqkv.data_ptr(), None if bqkv is None else bqkv.data_ptr(),
                               q.data_ptr(), k.data_ptr(), vt.data_ptr(), vt.shape[1], cos.data_ptr(),
                               sin.data_ptr(), pos0, M, n_q_heads, n_kv_heads, head_dim, K, q_scale, _stream()))
    return q, k, vt


# ---- host-side scheduler ------------------------------------------------------------------------

class Scheduler:
    """A po_sched: SRJF with continuous JCT calibration (same names as the C ABI)."""

    def __init__(self, lam: float):
        h = C.c_void_p()
        check(lib().po_sched_create(lam, C.byref(h)))
        self._h = h

    def po_sched_set_jct_model(self, c0: float, c_input: float, c_cached: float) -> None:
        check(lib().po_sched_set_jct_model(self._h, c0, c_input, c_cached))

    def po_sched_fit_jct_model(self, n_input, n_cached, jct):
        a = np.ascontiguousarray(n_input, dtype=np.int64)
        b = np.ascontiguousarray(n_cached, dtype=np.int64)
        z = np.ascontiguousarray(jct, dtype=np.float64)
        coef = (C.c_double * 3)()
        check(lib().po_sched_fit_jct_model(self._h, _host_ptr(a), _host_ptr(b), _host_ptr(z), len(a), C.byref(coef)))
        return tuple(coef)

    def po_sched_push(self, rid: int, tokens, arrival_time: float) -> None:
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        check(lib().po_sched_push(self._h, rid, _host_ptr(t), t.shape[0], arrival_time))

    def po_sched_push_request(self, rid: int, tokens, cand, arrival_time: float) -> None:
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        c = np.ascontiguousarray(cand, dtype=np.int32)
        check(lib().po_sched_push_request(self._h, rid, _host_ptr(t), t.shape[0], _host_ptr(c) if c.size else None, c.shape[0],
                                          arrival_time))

    def po_sched_size(self) -> int:
        return int(lib().po_sched_size(self._h))

    def po_sched_remove(self, rid: int) -> None:
        check(lib().po_sched_remove(self._h, rid))

    def po_sched_pick(self, cached_tokens, now: float):
        """-> (id or -1, tokens of that request that hit the prefix cache)"""
        c = np.ascontiguousarray(cached_tokens, dtype=np.int32)
        rid, hit = C.c_int64(-1), C.c_int64(0)
        check(lib().po_sched_pick(self._h, _host_ptr(c) if c.size else None, c.shape[0], now, C.byref(rid), C.byref(hit)))
        return rid.value, hit.value

    def po_sched_pick_multi(self, cached_entries, now: float):
        """po_sched_pick against several cache entries (a list of token-id arrays)."""
        ents = [np.ascontiguousarray(e, dtype=np.int32) for e in cached_entries]
        n = len(ents)
        ptrs = (C.c_void_p * max(n, 1))(*[e.ctypes.data if e.size else None for e in ents])
        lens = (C.c_int64 * max(n, 1))(*[e.shape[0] for e in ents])
        rid, hit = C.c_int64(-1), C.c_int64(0)
        check(lib().po_sched_pick_multi(self._h, ptrs, lens, n, now, C.byref(rid), C.byref(hit)))
        return rid.value, hit.value

    def po_sched_destroy(self) -> None:
        if getattr(self, "_h", None):
            lib().po_sched_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.po_sched_destroy()
        except Exception:
            pass
