"""ctypes binding of librelaygr.so: argument marshalling only.

Every function named relaygr_* below forwards to the C entry point of the same
name (include/relaygr.h).  PyTorch supplies device memory and the current HIP
stream; no step of the path runs in Python or in PyTorch ops.  If the library
is missing it is built once with hipcc; if that fails the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

from . import build as _build

RELAYGR_OK, RELAYGR_EINVAL, RELAYGR_ENOSPC, RELAYGR_ENOENT, RELAYGR_EHIP, RELAYGR_EBUSY = 0, -1, -2, -3, -4, -5
RELAYGR_TRIGGER_NOT_AT_RISK, RELAYGR_TRIGGER_ADMIT, RELAYGR_TRIGGER_REFUSED = 0, 1, 2
RELAYGR_DTYPE_FP32, RELAYGR_DTYPE_BF16, RELAYGR_DTYPE_FP16 = 0, 1, 2
RELAYGR_NO_CACHE = 0
RELAYGR_TILE_TOKENS = 64

EXPORTS = [
    "relaygr_kv_footprint_bytes", "relaygr_kv_pool_bytes_for", "relaygr_scratch_bytes",
    "relaygr_ctx_create", "relaygr_ctx_destroy", "relaygr_ctx_set_attention",
    "relaygr_kv_pool_create", "relaygr_kv_pool_destroy", "relaygr_kv_pool_alloc", "relaygr_kv_pool_free",
    "relaygr_kv_pool_lookup", "relaygr_kv_pool_entry_len", "relaygr_kv_pool_stats", "relaygr_kv_pool_locate",
    "relaygr_prefill_prefix", "relaygr_rank_with_cache", "relaygr_rank_full_recompute",
    "relaygr_rank_with_cache_static", "relaygr_static_scratch_bytes",
    "relaygr_ctx_profile_enable", "relaygr_ctx_profile_sample", "relaygr_ctx_profile_read",
    "relaygr_kv_pool_entry_bytes", "relaygr_kv_pool_spill", "relaygr_kv_pool_reload",
    "relaygr_expander_create", "relaygr_expander_destroy", "relaygr_expander_retire",
    "relaygr_expander_alloc", "relaygr_expander_trim", "relaygr_expander_lookup", "relaygr_expander_stats",
    "relaygr_expander_set_reload_rate",
    "relaygr_admission_budget_compute", "relaygr_slot_throughput",
    "relaygr_trigger_create", "relaygr_trigger_destroy", "relaygr_trigger_admit", "relaygr_trigger_release",
    "relaygr_trigger_stats",
    "relaygr_last_error",
]
EXPANDER_STATS = ["hbm_hits", "dram_hits", "misses", "refusals", "spills", "dram_evictions", "dram_bytes", "dram_entries",
                  "hbm_evictions", "hbm_reclaimable"]
KERNEL_CLASSES = ["setup", "ln", "f1", "attn", "gate", "f2", "score"]


class ModelConfigC(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("dtype", C.c_int32), ("ln_eps", C.c_float)]


class LayerWeightsC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("ln_in_g", "ln_in_b", "w1", "b1", "ln_at_g", "ln_at_b", "w2", "b2")]


class WeightsC(C.Structure):
    _fields_ = [("layers", C.POINTER(LayerWeightsC)), ("ln_out_g", C.c_void_p), ("ln_out_b", C.c_void_p),
                ("w_score", C.c_void_p), ("b_score", C.c_float)]


class BatchC(C.Structure):
    _fields_ = [("n_users", C.c_int32),
                ("user_ids", C.POINTER(C.c_uint64)),
                ("handles", C.POINTER(C.c_uint64)),
                ("prefix_emb", C.c_void_p), ("prefix_off", C.POINTER(C.c_int32)),
                ("suffix_emb", C.c_void_p), ("suffix_off", C.POINTER(C.c_int32)),
                ("cand_emb", C.c_void_p), ("cand_off", C.POINTER(C.c_int32))]


class AdmissionParamsC(C.Structure):
    _fields_ = [("q_m", C.c_double), ("model_slots", C.c_int32), ("kv_p99_bytes", C.c_double),
                ("hbm_bytes", C.c_double), ("r1", C.c_double), ("n_instances", C.c_int32),
                ("r2", C.c_double), ("t_life_s", C.c_double)]


class AdmissionBudgetC(C.Structure):
    _fields_ = [(n, C.c_double) for n in
                ("max_live_caches", "q_admit_hbm", "q_admit_compute", "q_admit", "q_max")]


class RelayGRError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"relaygr error {code}: {message}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Loads librelaygr.so from the package directory (building it first if it is absent)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    lib = C.CDLL(_build.LIB)
    vp, i32, i64, u64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_size_t
    P = C.POINTER
    sig = {
        "relaygr_kv_footprint_bytes": (sz, [P(ModelConfigC), i32]),
        "relaygr_kv_pool_bytes_for": (sz, [P(ModelConfigC), i32, i32]),
        "relaygr_scratch_bytes": (sz, [P(ModelConfigC), i32, i64, i64]),
        "relaygr_ctx_create": (C.c_int, [P(ModelConfigC), P(WeightsC), vp, sz, P(vp)]),
        "relaygr_ctx_destroy": (None, [vp]),
        "relaygr_kv_pool_create": (C.c_int, [P(ModelConfigC), vp, sz, i32, P(vp)]),
        "relaygr_kv_pool_destroy": (None, [vp]),
        "relaygr_kv_pool_alloc": (C.c_int, [vp, u64, i32, P(u64)]),
        "relaygr_kv_pool_free": (C.c_int, [vp, u64]),
        "relaygr_kv_pool_lookup": (C.c_int, [vp, u64, P(u64)]),
        "relaygr_kv_pool_entry_len": (C.c_int, [vp, u64, P(i32)]),
        "relaygr_kv_pool_stats": (C.c_int, [vp, P(i64), P(i64), P(i64), P(i64)]),
        "relaygr_kv_pool_locate": (C.c_int, [vp, u64, i32, i32, i32, P(i64), P(i64)]),
        "relaygr_prefill_prefix": (C.c_int, [vp, vp, P(BatchC), vp]),
        "relaygr_rank_with_cache": (C.c_int, [vp, vp, P(BatchC), vp, vp]),
        "relaygr_rank_full_recompute": (C.c_int, [vp, P(BatchC), vp, vp]),
        "relaygr_rank_with_cache_static": (C.c_int, [vp, vp, P(BatchC), vp, vp]),
        "relaygr_static_scratch_bytes": (sz, []),
        "relaygr_ctx_profile_enable": (C.c_int, [vp, C.c_uint32]),
        "relaygr_ctx_profile_sample": (C.c_int, [vp, i32]),
        "relaygr_ctx_set_attention": (C.c_int, [vp, i32]),
        "relaygr_ctx_profile_read": (C.c_int, [vp, i32, P(C.c_double), P(i64)]),
        "relaygr_kv_pool_entry_bytes": (sz, [vp, u64]),
        "relaygr_kv_pool_spill": (C.c_int, [vp, u64, vp, sz, vp]),
        "relaygr_kv_pool_reload": (C.c_int, [vp, u64, i32, vp, sz, vp, P(u64)]),
        "relaygr_expander_create": (C.c_int, [vp, sz, i32, P(vp)]),
        "relaygr_expander_destroy": (None, [vp]),
        "relaygr_expander_retire": (C.c_int, [vp, u64, vp]),
        "relaygr_expander_alloc": (C.c_int, [vp, u64, i32, P(u64)]),
        "relaygr_expander_trim": (C.c_int, [vp, i32]),
        "relaygr_expander_set_reload_rate": (C.c_int, [vp, C.c_double, C.c_double]),
        "relaygr_expander_lookup": (C.c_int, [vp, u64, vp, P(u64), P(i32)]),
        "relaygr_expander_stats": (C.c_int, [vp, P(i64)]),
        "relaygr_admission_budget_compute": (C.c_int, [P(AdmissionParamsC), P(AdmissionBudgetC)]),
        "relaygr_slot_throughput": (C.c_double, [C.c_double]),
        "relaygr_trigger_create": (C.c_int, [P(AdmissionBudgetC), i32, P(vp)]),
        "relaygr_trigger_destroy": (None, [vp]),
        "relaygr_trigger_admit": (C.c_int, [vp, C.c_double, i32]),
        "relaygr_trigger_release": (C.c_int, [vp]),
        "relaygr_trigger_stats": (C.c_int, [vp, P(i64), P(i64), P(i64), P(i64)]),
        "relaygr_last_error": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)   # AttributeError here means the library lacks a declared symbol
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != RELAYGR_OK:
        raise RelayGRError(rc, load_library().relaygr_last_error().decode("utf-8", "replace"))


def relaygr_last_error() -> str:
    return load_library().relaygr_last_error().decode("utf-8", "replace")


def _dtype_code(dtype: str) -> int:
    return {"fp32": RELAYGR_DTYPE_FP32, "bf16": RELAYGR_DTYPE_BF16, "fp16": RELAYGR_DTYPE_FP16}[dtype]


def _torch_dtype(dtype: str):
    return {"fp32": torch.float32, "bf16": torch.bfloat16, "fp16": torch.float16}[dtype]


def make_config(n_layers: int, d_model: int, n_heads: int, dtype: str, ln_eps: float = 1e-5) -> ModelConfigC:
    return ModelConfigC(n_layers, d_model, n_heads, _dtype_code(dtype), ln_eps)


def relaygr_kv_footprint_bytes(cfg: ModelConfigC, prefix_len: int) -> int:
    return load_library().relaygr_kv_footprint_bytes(C.byref(cfg), prefix_len)


def relaygr_kv_pool_bytes_for(cfg: ModelConfigC, prefix_len: int, page_tokens: int) -> int:
    return load_library().relaygr_kv_pool_bytes_for(C.byref(cfg), prefix_len, page_tokens)


def relaygr_scratch_bytes(cfg: ModelConfigC, max_users: int, max_prefix_tokens: int, max_new_tokens: int) -> int:
    return load_library().relaygr_scratch_bytes(C.byref(cfg), max_users, max_prefix_tokens, max_new_tokens)


def _stream_ptr(stream) -> int:
    """HIP stream handle of a torch stream (default: torch's current stream) or a raw hipStream_t given as an int."""
    if isinstance(stream, int):
        return stream
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


class Context:
    """relaygr_ctx plus the device tensors it references (weights, scratch)."""

    def __init__(self, model_cfg, weights: dict, max_users: int, max_prefix_tokens: int, max_new_tokens: int,
                 device: str = "cuda:0"):
        lib = load_library()
        self.dtype = model_cfg.dtype
        self.cfg = make_config(model_cfg.n_layers, model_cfg.d_model, model_cfg.n_heads, model_cfg.dtype, model_cfg.ln_eps)
        td = _torch_dtype(self.dtype)
        self.device = torch.device(device)
        self._keep = []

        def dev(a):
            t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device).to(td).contiguous()
            self._keep.append(t)
            return t.data_ptr()

        layers = (LayerWeightsC * model_cfg.n_layers)()
        for l, lw in enumerate(weights["layers"]):
            for name, _ in LayerWeightsC._fields_:
                setattr(layers[l], name, dev(lw[name]))
        self._layers = layers
        wc = WeightsC(layers, dev(weights["ln_out_g"]), dev(weights["ln_out_b"]), dev(weights["w_score"]),
                      float(weights["b_score"]))
        nbytes = relaygr_scratch_bytes(self.cfg, max_users, max_prefix_tokens, max_new_tokens)
        if nbytes == 0:
            raise RelayGRError(RELAYGR_EINVAL, "relaygr_scratch_bytes rejected the configuration")
        self.scratch = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.scratch_bytes = nbytes
        h = C.c_void_p()
        _check(lib.relaygr_ctx_create(C.byref(self.cfg), C.byref(wc), self.scratch.data_ptr(), nbytes, C.byref(h)))
        self.handle = h
        form = getattr(model_cfg, "attention", "silu")
        if form != "silu":
            relaygr_ctx_set_attention(self, form)

    def close(self):
        if getattr(self, "handle", None):
            torch.cuda.synchronize(self.device)
            load_library().relaygr_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


ATTENTION_FORMS = {"silu": 0, "softmax": 1}


def relaygr_ctx_set_attention(ctx: Context, form: str) -> None:
    """Selects the context's attention form: "silu" (pointwise SiLU, the default) or "softmax"."""
    if form not in ATTENTION_FORMS:
        raise RelayGRError(RELAYGR_EINVAL, f"unknown attention form {form!r}")
    _check(load_library().relaygr_ctx_set_attention(ctx.handle, ATTENTION_FORMS[form]))


def relaygr_ctx_profile_enable(ctx: Context, classes: Sequence[str]) -> None:
    mask = 0
    for c in classes:
        mask |= 1 << KERNEL_CLASSES.index(c)
    _check(load_library().relaygr_ctx_profile_enable(ctx.handle, mask))


def relaygr_ctx_profile_sample(ctx: Context, every_n_calls: int) -> None:
    _check(load_library().relaygr_ctx_profile_sample(ctx.handle, every_n_calls))


def relaygr_ctx_profile_read(ctx: Context, kernel_class: str):
    """(total milliseconds, launches) of one kernel class since profiling was enabled."""
    ms, n = C.c_double(), C.c_int64()
    _check(load_library().relaygr_ctx_profile_read(ctx.handle, KERNEL_CLASSES.index(kernel_class), C.byref(ms), C.byref(n)))
    return ms.value, n.value


class KvPool:
    """relaygr_kv_pool over a torch-allocated device slab."""

    def __init__(self, cfg: ModelConfigC, dtype: str, slab_bytes: int, page_tokens: int = 256, device: str = "cuda:0"):
        lib = load_library()
        self.cfg = cfg
        self.dtype = dtype
        self.device = torch.device(device)
        self.slab = torch.empty(slab_bytes, dtype=torch.uint8, device=self.device)
        h = C.c_void_p()
        _check(lib.relaygr_kv_pool_create(C.byref(cfg), self.slab.data_ptr(), slab_bytes, page_tokens, C.byref(h)))
        self.handle = h

    def elements(self) -> torch.Tensor:
        """The slab viewed in the storage dtype (for inspection with relaygr_kv_pool_locate)."""
        return self.slab.view(_torch_dtype(self.dtype))

    def close(self):
        if getattr(self, "handle", None):
            load_library().relaygr_kv_pool_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def relaygr_kv_pool_alloc(pool: KvPool, user_id: int, prefix_len: int) -> int:
    out = C.c_uint64(0)
    _check(load_library().relaygr_kv_pool_alloc(pool.handle, user_id, prefix_len, C.byref(out)))
    return out.value


def relaygr_kv_pool_free(pool: KvPool, handle: int) -> None:
    _check(load_library().relaygr_kv_pool_free(pool.handle, handle))


def relaygr_kv_pool_lookup(pool: KvPool, user_id: int) -> int:
    """Handle of the user's live entry, or RELAYGR_NO_CACHE if there is none."""
    out = C.c_uint64(0)
    rc = load_library().relaygr_kv_pool_lookup(pool.handle, user_id, C.byref(out))
    if rc == RELAYGR_ENOENT:
        return RELAYGR_NO_CACHE
    _check(rc)
    return out.value


def relaygr_kv_pool_entry_len(pool: KvPool, handle: int) -> int:
    out = C.c_int32(0)
    _check(load_library().relaygr_kv_pool_entry_len(pool.handle, handle, C.byref(out)))
    return out.value


def relaygr_kv_pool_stats(pool: KvPool) -> dict:
    a, b, c, d = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
    _check(load_library().relaygr_kv_pool_stats(pool.handle, C.byref(a), C.byref(b), C.byref(c), C.byref(d)))
    return {"pages_total": a.value, "pages_free": b.value, "live_entries": c.value, "largest_free_extent": d.value}


def relaygr_kv_pool_locate(pool: KvPool, handle: int, layer: int, token: int, feature: int):
    k, v = C.c_int64(), C.c_int64()
    _check(load_library().relaygr_kv_pool_locate(pool.handle, handle, layer, token, feature, C.byref(k), C.byref(v)))
    return k.value, v.value


# ---- DRAM tier -------------------------------------------------------------------------------
def relaygr_kv_pool_entry_bytes(pool: KvPool, handle: int) -> int:
    return load_library().relaygr_kv_pool_entry_bytes(pool.handle, handle)


def relaygr_kv_pool_spill(pool: KvPool, handle: int, host: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Enqueues the copy of the entry's extent into a pinned uint8 host tensor (made here if not given)."""
    n = relaygr_kv_pool_entry_bytes(pool, handle)
    if host is None:
        host = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    _check(load_library().relaygr_kv_pool_spill(pool.handle, handle, host.data_ptr(), host.numel(), _stream_ptr(stream)))
    return host


def relaygr_kv_pool_reload(pool: KvPool, user_id: int, prefix_len: int, host: torch.Tensor, stream=None) -> int:
    out = C.c_uint64(0)
    _check(load_library().relaygr_kv_pool_reload(pool.handle, user_id, prefix_len, host.data_ptr(), host.numel(),
                                                 _stream_ptr(stream), C.byref(out)))
    return out.value


class Expander:
    """relaygr_expander over a KvPool."""

    def __init__(self, pool: KvPool, dram_budget_bytes: int, max_inflight_reloads: int = 4):
        self.pool = pool
        h = C.c_void_p()
        _check(load_library().relaygr_expander_create(pool.handle, dram_budget_bytes, max_inflight_reloads, C.byref(h)))
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            load_library().relaygr_expander_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def relaygr_expander_retire(ex: Expander, handle: int, stream=None) -> None:
    _check(load_library().relaygr_expander_retire(ex.handle, handle, _stream_ptr(stream)))


def relaygr_expander_alloc(ex: Expander, user_id: int, prefix_len: int) -> int:
    out = C.c_uint64(0)
    _check(load_library().relaygr_expander_alloc(ex.handle, user_id, prefix_len, C.byref(out)))
    return out.value


def relaygr_expander_set_reload_rate(ex: Expander, bytes_per_second: float, burst_bytes: float) -> None:
    _check(load_library().relaygr_expander_set_reload_rate(ex.handle, C.c_double(bytes_per_second), C.c_double(burst_bytes)))


def relaygr_expander_trim(ex: Expander, keep: int = 0) -> None:
    _check(load_library().relaygr_expander_trim(ex.handle, keep))


def relaygr_expander_lookup(ex: Expander, user_id: int, stream=None):
    """(handle, source) with source 0 = HBM, 1 = reloaded from DRAM; raises RelayGRError with code
    RELAYGR_ENOENT (in neither tier) or RELAYGR_EBUSY (reload limit reached)."""
    out, src = C.c_uint64(0), C.c_int32(-1)
    _check(load_library().relaygr_expander_lookup(ex.handle, user_id, _stream_ptr(stream), C.byref(out), C.byref(src)))
    return out.value, src.value


def relaygr_expander_stats(ex: Expander) -> dict:
    a = (C.c_int64 * 10)()
    _check(load_library().relaygr_expander_stats(ex.handle, a))
    return dict(zip(EXPANDER_STATS, list(a)))


# ---- sequence-aware trigger (host arithmetic only) ---------------------------------------------
def relaygr_admission_budget_compute(q_m: float, model_slots: int, kv_p99_bytes: float, hbm_bytes: float, r1: float,
                                     n_instances: int, r2: float, t_life_s: float) -> dict:
    p = AdmissionParamsC(q_m, model_slots, kv_p99_bytes, hbm_bytes, r1, n_instances, r2, t_life_s)
    b = AdmissionBudgetC()
    _check(load_library().relaygr_admission_budget_compute(C.byref(p), C.byref(b)))
    return {n: getattr(b, n) for n, _ in AdmissionBudgetC._fields_}


def relaygr_slot_throughput(pre_infer_ms: float) -> float:
    return load_library().relaygr_slot_throughput(pre_infer_ms)


class Trigger:
    """relaygr_trigger: the admission gate of one special instance."""

    def __init__(self, budget: dict, len_threshold: int):
        b = AdmissionBudgetC(*[budget[n] for n, _ in AdmissionBudgetC._fields_])
        h = C.c_void_p()
        _check(load_library().relaygr_trigger_create(C.byref(b), len_threshold, C.byref(h)))
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            load_library().relaygr_trigger_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def relaygr_trigger_admit(t: Trigger, now_s: float, prefix_len: int) -> int:
    rc = load_library().relaygr_trigger_admit(t.handle, now_s, prefix_len)
    if rc < 0:
        _check(rc)
    return rc


def relaygr_trigger_release(t: Trigger) -> None:
    _check(load_library().relaygr_trigger_release(t.handle))


def relaygr_trigger_stats(t: Trigger) -> dict:
    a, b, c, d = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
    load_library().relaygr_trigger_stats(t.handle, C.byref(a), C.byref(b), C.byref(c), C.byref(d))
    return {"live": a.value, "admitted": b.value, "refused": c.value, "not_at_risk": d.value}


class Batch:
    """Device embeddings + host offsets of one jagged batch, marshalled as relaygr_batch."""

    def __init__(self, batch: dict, dtype: str, device: str = "cuda:0", handles: Optional[Sequence[int]] = None):
        td = _torch_dtype(dtype)
        self.n_users = int(batch["n_users"])
        dv = torch.device(device)

        def emb(a):
            if isinstance(a, torch.Tensor):
                return a
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dv).to(td).contiguous()

        self.prefix_emb = emb(batch["prefix_emb"])
        self.suffix_emb = emb(batch["suffix_emb"])
        self.cand_emb = emb(batch["cand_emb"])
        self.prefix_off = np.ascontiguousarray(batch["prefix_off"], dtype=np.int32)
        self.suffix_off = np.ascontiguousarray(batch["suffix_off"], dtype=np.int32)
        self.cand_off = np.ascontiguousarray(batch["cand_off"], dtype=np.int32)
        self.user_ids = np.ascontiguousarray(batch["user_ids"], dtype=np.uint64)
        self.handles = np.zeros(self.n_users, dtype=np.uint64)
        if handles is not None:
            self.set_handles(handles)
        self.n_cands = int(self.cand_off[-1]) if self.n_users else 0

    def set_handles(self, handles: Sequence[int]) -> None:
        self.handles = np.ascontiguousarray(np.asarray(handles, dtype=np.uint64))

    def c_struct(self) -> BatchC:
        def ptr(t):
            return t.data_ptr() if t.numel() else None
        return BatchC(
            self.n_users,
            self.user_ids.ctypes.data_as(C.POINTER(C.c_uint64)),
            self.handles.ctypes.data_as(C.POINTER(C.c_uint64)),
            ptr(self.prefix_emb), self.prefix_off.ctypes.data_as(C.POINTER(C.c_int32)),
            ptr(self.suffix_emb), self.suffix_off.ctypes.data_as(C.POINTER(C.c_int32)),
            ptr(self.cand_emb), self.cand_off.ctypes.data_as(C.POINTER(C.c_int32)),
        )


def relaygr_prefill_prefix(ctx: Context, pool: KvPool, batch: Batch, stream=None) -> None:
    bc = batch.c_struct()
    _check(load_library().relaygr_prefill_prefix(ctx.handle, pool.handle, C.byref(bc), _stream_ptr(stream)))


def relaygr_rank_with_cache(ctx: Context, pool: Optional[KvPool], batch: Batch, scores: Optional[torch.Tensor] = None,
                            stream=None) -> torch.Tensor:
    if scores is None:
        scores = torch.empty(batch.n_cands, dtype=torch.float32, device=ctx.device)
    bc = batch.c_struct()
    _check(load_library().relaygr_rank_with_cache(ctx.handle, pool.handle if pool is not None else None, C.byref(bc),
                                                  scores.data_ptr(), _stream_ptr(stream)))
    return scores


def relaygr_rank_with_cache_static(ctx: Context, pool: Optional[KvPool], batch: Batch, scores: torch.Tensor, stream=None) -> torch.Tensor:
    """relaygr_rank_with_cache on the library's own scratch; `scores` must be given (nothing is allocated)."""
    bc = batch.c_struct()
    _check(load_library().relaygr_rank_with_cache_static(ctx.handle, pool.handle if pool is not None else None, C.byref(bc),
                                                         scores.data_ptr(), _stream_ptr(stream)))
    return scores


def relaygr_static_scratch_bytes() -> int:
    return load_library().relaygr_static_scratch_bytes()


def relaygr_rank_full_recompute(ctx: Context, batch: Batch, scores: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if scores is None:
        scores = torch.empty(batch.n_cands, dtype=torch.float32, device=ctx.device)
    bc = batch.c_struct()
    _check(load_library().relaygr_rank_full_recompute(ctx.handle, C.byref(bc), scores.data_ptr(), _stream_ptr(stream)))
    return scores
