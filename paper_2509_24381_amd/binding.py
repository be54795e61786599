"""ctypes binding of the C ABI in include/rserve_prefill.h.

Argument marshalling only: every step of the layer runs in the HIP library.  PyTorch is used for device
memory (`torch.empty(..., device="cuda")`, `.data_ptr()`) and for the current HIP stream; nothing here
computes.  If the shared library is missing the import of this module still works, but every use raises
RsError: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "librserve_prefill.so"

STATUS = {0: "RS_OK", -1: "RS_EINVAL", -2: "RS_ECAPACITY", -3: "RS_EWORKSPACE", -4: "RS_ESTATE", -5: "RS_EHIP"}

# every symbol include/rserve_prefill.h declares
EXPORTED_SYMBOLS = (
    "rs_ctx_create", "rs_ctx_destroy", "rs_weights_packed_bytes", "rs_weights_pack", "rs_kv_bytes", "rs_kv_alloc",
    "rs_kv_free", "rs_kv_len", "rs_kv_capacity", "rs_kv_reset", "rs_kv_truncate", "rs_kv_export", "rs_kv_import",
    "rs_kv_page_bytes", "rs_kv_pool_create", "rs_kv_pool_destroy", "rs_kv_pool_pages", "rs_kv_pool_free_pages",
    "rs_kv_alloc_paged",
    "rs_kv_fp8_bytes", "rs_kv_alloc_fp8", "rs_kv_is_fp8", "rs_kv_export_codes", "rs_kv_import_codes", "rs_workspace_bytes_fp8kv",
    "rs_kv_page_bytes_fp8", "rs_kv_pool_create_fp8", "rs_kv_pool_is_fp8", "rs_kv_alloc_paged_fp8",
    "rs_workspace_bytes", "rs_prefill_chunk", "rs_prefill_chunk_static", "rs_static_workspace_bytes", "rs_prefill_batch", "rs_prefill_model_batch", "rs_prefill_model_batch_mrope", "rs_ctx_set_mrope_sections",
    "rs_prefill_batch_mrope", "rs_lm_head_workspace_bytes",
    "rs_lm_head", "rs_last_error", "rs_version",
    "rs_profile_enable", "rs_profile_sample_every", "rs_profile_read",
)

SCHED_SYMBOLS = (
    "rs_sched_create", "rs_sched_destroy", "rs_sched_add_request", "rs_sched_mark_ready", "rs_sched_schedulable_tokens",
    "rs_sched_prompt_length", "rs_sched_prefilled_tokens", "rs_sched_encoder_batches", "rs_sched_next_round",
    "rs_sched_queue_length", "rs_sched_queue_ids", "rs_sched_release_request",
)

STEPS = ("row_rms", "qkv_gemm", "append_kv", "attention", "o_gemm", "gate_up_gemm", "down_gemm")


class RsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status
        self.status_name = STATUS.get(status, str(status))


class _Cfg(C.Structure):
    _fields_ = [("hidden", C.c_int), ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int),
                ("mlp_inter", C.c_int), ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("qkv_bias", C.c_int),
                ("max_tokens_per_call", C.c_int), ("max_requests", C.c_int), ("max_pos", C.c_int)]


class _Segment(C.Structure):
    _fields_ = [("is_mm", C.c_int), ("n_tokens", C.c_int)]


class _RoundEntry(C.Structure):
    _fields_ = [("request_id", C.c_int64), ("first_token", C.c_int), ("n_tokens", C.c_int), ("finished", C.c_int)]


class _EncodeBatch(C.Structure):
    _fields_ = [("first_segment", C.c_int), ("last_segment", C.c_int), ("n_items", C.c_int), ("n_tokens", C.c_int)]


class _Weights(C.Structure):
    _fields_ = [("ln1_g", C.c_void_p), ("w_qkv", C.c_void_p), ("b_qkv", C.c_void_p), ("w_o", C.c_void_p),
                ("ln2_g", C.c_void_p), ("w_gate_up", C.c_void_p), ("w_down", C.c_void_p)]


_lib = None


def library_path() -> str:
    return os.path.join(PKG_DIR, _LIB_NAME)


def load_library():
    """Loads librserve_prefill.so (built in-tree by paper_2509_24381_amd.build) and declares the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RsError(-5, f"{path} is not built; run `python -m paper_2509_24381_amd.build` (there is no fallback path)")
    lib = C.CDLL(path)
    vp, sz, i = C.c_void_p, C.c_size_t, C.c_int
    proto = {
        "rs_ctx_create": (i, [C.POINTER(_Cfg), C.POINTER(vp)]),
        "rs_ctx_destroy": (None, [vp]),
        "rs_weights_packed_bytes": (sz, [vp]),
        "rs_weights_pack": (i, [vp, C.POINTER(_Weights), vp, sz, C.POINTER(_Weights), vp]),
        "rs_kv_bytes": (sz, [vp, i, i]),
        "rs_kv_alloc": (i, [vp, i, i, vp, sz, C.POINTER(vp)]),
        "rs_kv_free": (None, [vp]),
        "rs_kv_len": (i, [vp, i]),
        "rs_kv_capacity": (i, [vp]),
        "rs_kv_reset": (i, [vp]),
        "rs_kv_truncate": (i, [vp, i, i]),
        "rs_kv_export": (i, [vp, i, vp, vp, vp]),
        "rs_kv_import": (i, [vp, i, vp, vp, i, vp]),
        "rs_kv_page_bytes": (sz, [vp]),
        "rs_kv_pool_create": (i, [vp, vp, sz, C.POINTER(vp)]),
        "rs_kv_pool_destroy": (i, [vp]),
        "rs_kv_pool_pages": (i, [vp]),
        "rs_kv_pool_free_pages": (i, [vp]),
        "rs_kv_alloc_paged": (i, [vp, vp, i, C.POINTER(vp)]),
        "rs_workspace_bytes": (sz, [vp, i, i]),
        "rs_kv_fp8_bytes": (sz, [vp, i, i]),
        "rs_kv_alloc_fp8": (i, [vp, i, i, C.c_float, C.c_float, vp, sz, C.POINTER(vp)]),
        "rs_kv_is_fp8": (i, [vp]),
        "rs_kv_export_codes": (i, [vp, i, vp, vp, vp]),
        "rs_kv_import_codes": (i, [vp, i, vp, vp, i, vp]),
        "rs_workspace_bytes_fp8kv": (sz, [vp, i, i, sz]),
        "rs_kv_page_bytes_fp8": (sz, [vp]),
        "rs_kv_pool_create_fp8": (i, [vp, vp, sz, C.POINTER(vp)]),
        "rs_kv_pool_is_fp8": (i, [vp]),
        "rs_kv_alloc_paged_fp8": (i, [vp, vp, i, C.c_float, C.c_float, C.POINTER(vp)]),
        "rs_prefill_chunk": (i, [vp, C.POINTER(_Weights), i, vp, vp, i, vp, vp, sz, vp]),
        "rs_prefill_chunk_static": (i, [vp, C.POINTER(_Weights), i, vp, vp, i, vp, vp]),
        "rs_static_workspace_bytes": (sz, []),
        "rs_prefill_batch": (i, [vp, C.POINTER(_Weights), i, C.POINTER(vp), C.POINTER(i), i, vp, vp, vp, sz, vp]),
        "rs_prefill_model_batch": (i, [vp, C.POINTER(_Weights), i, C.POINTER(vp), C.POINTER(i), i, vp, vp, vp, sz, vp]),
        "rs_prefill_model_batch_mrope": (i, [vp, C.POINTER(_Weights), i, C.POINTER(vp), C.POINTER(i), i, C.POINTER(i), vp, vp, vp, sz, vp]),
        "rs_ctx_set_mrope_sections": (i, [vp, i, i, i]),
        "rs_prefill_batch_mrope": (i, [vp, C.POINTER(_Weights), i, C.POINTER(vp), C.POINTER(i), i, C.POINTER(i), vp, vp, vp, sz, vp]),
        "rs_lm_head_workspace_bytes": (sz, [vp, i]),
        "rs_lm_head": (i, [vp, vp, vp, i, vp, i, vp, vp, sz, vp]),
        "rs_last_error": (C.c_char_p, []),
        "rs_version": (i, []),
        "rs_profile_enable": (i, [vp, i, i]),
        "rs_profile_sample_every": (i, [vp, i]),
        "rs_profile_read": (i, [vp, C.POINTER(C.c_double), C.POINTER(i)]),
        "rs_sched_create": (i, [i, C.POINTER(vp)]),
        "rs_sched_destroy": (None, [vp]),
        "rs_sched_add_request": (i, [vp, C.c_int64, C.POINTER(_Segment), i]),
        "rs_sched_mark_ready": (i, [vp, C.c_int64, i]),
        "rs_sched_schedulable_tokens": (i, [vp, C.c_int64]),
        "rs_sched_prompt_length": (i, [vp, C.c_int64]),
        "rs_sched_prefilled_tokens": (i, [vp, C.c_int64]),
        "rs_sched_encoder_batches": (i, [vp, C.c_int64, i, C.POINTER(_EncodeBatch), i, C.POINTER(i)]),
        "rs_sched_next_round": (i, [vp, C.POINTER(_RoundEntry), i, C.POINTER(i)]),
        "rs_sched_queue_length": (i, [vp]),
        "rs_sched_queue_ids": (i, [vp, C.POINTER(C.c_int64), i, C.POINTER(i)]),
        "rs_sched_release_request": (i, [vp, C.c_int64]),
    }
    for name, (res, args) in proto.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise RsError(status, load_library().rs_last_error().decode("utf-8", "replace"))


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream_handle(stream) -> Optional[int]:
    import torch
    if isinstance(stream, int):
        return stream or None
    if stream is None:
        if not torch.cuda.is_available():
            return None  # GPU-less host: the call can only reach the library's argument checks
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) or None


@dataclass
class LayerConfig:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp_inter: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    qkv_bias: bool = False
    max_tokens_per_call: int = 4096
    max_requests: int = 64
    max_pos: int = 32768

    def _c(self) -> _Cfg:
        return _Cfg(self.hidden, self.n_q_heads, self.n_kv_heads, self.head_dim, self.mlp_inter, self.rms_eps,
                    self.rope_theta, int(self.qkv_bias), self.max_tokens_per_call, self.max_requests, self.max_pos)


class PackedWeights:
    """One layer's weights in the library's packed layout; owns the device slab."""

    def __init__(self, slab, struct: _Weights):
        self.slab = slab
        self.struct = struct


class KVPool:
    """A pool of KV pages (64 tokens of one layer each) in one device slab; paged caches take their pages from it."""

    def __init__(self, ctx: "Context", n_pages: int, fp8: bool = False):
        import torch
        self.ctx = ctx
        self.fp8 = fp8
        self.page_bytes = (ctx.lib.rs_kv_page_bytes_fp8 if fp8 else ctx.lib.rs_kv_page_bytes)(ctx.handle)
        self.slab = torch.empty(max(n_pages * self.page_bytes, 256), dtype=torch.uint8, device="cuda")
        h = C.c_void_p()
        create = ctx.lib.rs_kv_pool_create_fp8 if fp8 else ctx.lib.rs_kv_pool_create
        _check(create(ctx.handle, _ptr(self.slab), n_pages * self.page_bytes, C.byref(h)))
        self.handle = h

    def __del__(self):
        try:
            if self.handle:
                load_library().rs_kv_pool_destroy(self.handle)   # refuses (and leaks the handle) while caches are alive
                self.handle = None
        except Exception:
            pass

    @property
    def pages(self) -> int:
        return load_library().rs_kv_pool_pages(self.handle)

    @property
    def free_pages(self) -> int:
        return load_library().rs_kv_pool_free_pages(self.handle)

    def new_cache(self, n_layers: int, k_scale: float = 1.0, v_scale: float = 1.0) -> "KVCache":
        """An empty growable cache on this pool (the scales matter for a pool of 8-bit pages only)."""
        h = C.c_void_p()
        if self.fp8:
            _check(self.ctx.lib.rs_kv_alloc_paged_fp8(self.ctx.handle, self.handle, n_layers, k_scale, v_scale, C.byref(h)))
        else:
            _check(self.ctx.lib.rs_kv_alloc_paged(self.ctx.handle, self.handle, n_layers, C.byref(h)))
        return KVCache(self.ctx, h.value, self.slab, pool=self)


class KVCache:
    """One request's KV cache over n_layers layers; holds the device slab (its own, or its pool's) and the host handle."""

    def __init__(self, ctx: "Context", handle: int, slab, pool: "KVPool" = None):
        self.ctx = ctx
        self.handle = C.c_void_p(handle)
        self.slab = slab
        self.pool = pool          # keeps the pool alive as long as the cache

    def __del__(self):
        try:
            if self.handle:
                load_library().rs_kv_free(self.handle)
                self.handle = None
        except Exception:
            pass

    def length(self, layer: int = 0) -> int:
        return load_library().rs_kv_len(self.handle, layer)

    @property
    def capacity(self) -> int:
        return load_library().rs_kv_capacity(self.handle)

    def reset(self):
        _check(load_library().rs_kv_reset(self.handle))

    def truncate(self, layer: int, n_tokens: int):
        _check(load_library().rs_kv_truncate(self.handle, layer, n_tokens))

    def export(self, layer: int = 0, stream=None):
        """(K~, V) of `layer` as bf16 tensors [len, Hkv, d] on the device."""
        import torch
        n = self.length(layer)
        cfg = self.ctx.cfg
        k = torch.empty((n, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
        v = torch.empty_like(k)
        _check(load_library().rs_kv_export(self.handle, layer, _ptr(k) if n else None, _ptr(v) if n else None,
                                           _stream_handle(stream)))
        return k, v

    def import_(self, layer: int, k, v, stream=None):
        """Loads bf16 [n, Hkv, d] device tensors as the cache content of `layer`."""
        n = int(k.shape[0])
        assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
        _check(load_library().rs_kv_import(self.handle, layer, _ptr(k) if n else None, _ptr(v) if n else None, n,
                                           _stream_handle(stream)))

    @property
    def is_fp8(self) -> bool:
        return load_library().rs_kv_is_fp8(self.handle) == 1

    def export_codes(self, layer: int = 0, stream=None):
        """The stored bytes (K~, V) of an 8-bit cache's `layer` as uint8 tensors [len, Hkv, d] on the device."""
        import torch
        n = self.length(layer)
        cfg = self.ctx.cfg
        k = torch.empty((n, cfg.n_kv_heads, cfg.head_dim), dtype=torch.uint8, device="cuda")
        v = torch.empty_like(k)
        _check(load_library().rs_kv_export_codes(self.handle, layer, _ptr(k) if n else None, _ptr(v) if n else None,
                                                 _stream_handle(stream)))
        return k, v

    def import_codes(self, layer: int, k, v, stream=None):
        """Loads uint8 [n, Hkv, d] device tensors as the stored bytes of an 8-bit cache's `layer`."""
        n = int(k.shape[0])
        assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
        _check(load_library().rs_kv_import_codes(self.handle, layer, _ptr(k) if n else None, _ptr(v) if n else None, n,
                                                 _stream_handle(stream)))


class Context:
    def __init__(self, cfg: LayerConfig):
        self.cfg = cfg
        self.lib = load_library()
        h = C.c_void_p()
        c = cfg._c()
        _check(self.lib.rs_ctx_create(C.byref(c), C.byref(h)))
        self.handle = h

    def __del__(self):
        try:
            if getattr(self, "handle", None):
                self.lib.rs_ctx_destroy(self.handle)
                self.handle = None
        except Exception:
            pass

    # ---- sizes
    def weights_packed_bytes(self) -> int:
        return self.lib.rs_weights_packed_bytes(self.handle)

    def kv_bytes(self, n_layers: int, capacity: int) -> int:
        return self.lib.rs_kv_bytes(self.handle, n_layers, capacity)

    def workspace_bytes(self, max_tokens: int, max_requests: int = 1) -> int:
        return self.lib.rs_workspace_bytes(self.handle, max_tokens, max_requests)

    # ---- allocation helpers (device memory comes from torch)
    def pack_weights(self, ln1_g, w_qkv, w_o, ln2_g, w_gate_up, w_down, b_qkv=None, stream=None) -> PackedWeights:
        import torch
        src = _Weights(_ptr(ln1_g), _ptr(w_qkv), _ptr(b_qkv), _ptr(w_o), _ptr(ln2_g), _ptr(w_gate_up), _ptr(w_down))
        nbytes = self.weights_packed_bytes()
        slab = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        out = _Weights()
        _check(self.lib.rs_weights_pack(self.handle, C.byref(src), _ptr(slab), nbytes, C.byref(out), _stream_handle(stream)))
        return PackedWeights(slab, out)

    def kv_alloc(self, n_layers: int, capacity: int) -> KVCache:
        import torch
        nbytes = self.kv_bytes(n_layers, capacity)
        slab = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        h = C.c_void_p()
        _check(self.lib.rs_kv_alloc(self.handle, n_layers, capacity, _ptr(slab), nbytes, C.byref(h)))
        return KVCache(self, h.value, slab)

    def workspace(self, max_tokens: int, max_requests: int = 1, fp8_visible_tokens: int = 0):
        """Device workspace for calls of up to max_tokens rows and max_requests requests; with 8-bit caches also room for
        the bf16 expansion of fp8_visible_tokens tokens (cached + new, summed over a call's requests)."""
        import torch
        n = (self.lib.rs_workspace_bytes_fp8kv(self.handle, max_tokens, max_requests, fp8_visible_tokens)
             if fp8_visible_tokens else self.workspace_bytes(max_tokens, max_requests))
        return torch.empty(n, dtype=torch.uint8, device="cuda")

    def kv_alloc_fp8(self, n_layers: int, capacity: int, k_scale: float = 1.0, v_scale: float = 1.0) -> KVCache:
        """An 8-bit (E4M3) cache: value = decode(code) * scale."""
        import torch
        nbytes = self.lib.rs_kv_fp8_bytes(self.handle, n_layers, capacity)
        slab = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        h = C.c_void_p()
        _check(self.lib.rs_kv_alloc_fp8(self.handle, n_layers, capacity, k_scale, v_scale, _ptr(slab), nbytes, C.byref(h)))
        return KVCache(self, h.value, slab)

    # ---- measurement hook
    def profile_enable(self, step, max_launches: int = 1024, every: int = 1):
        """step: a name from STEPS, its index, or None / -1 to switch the hook off; every: measure each n-th launch."""
        idx = -1 if step is None else (STEPS.index(step) if isinstance(step, str) else int(step))
        _check(self.lib.rs_profile_sample_every(self.handle, every))
        _check(self.lib.rs_profile_enable(self.handle, idx, max_launches))

    def profile_read(self):
        """(total milliseconds, launches measured) since the hook was enabled or last read."""
        ms, n = C.c_double(), C.c_int()
        _check(self.lib.rs_profile_read(self.handle, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    # ---- the hot path
    def prefill_chunk(self, packed: PackedWeights, layer: int, kv: KVCache, x, y, workspace, stream=None):
        """One chunk of one request through one layer; x, y: bf16 [T, H] device tensors (y may be x)."""
        t = int(x.shape[0])
        _check(self.lib.rs_prefill_chunk(self.handle, C.byref(packed.struct), layer, kv.handle, _ptr(x), t, _ptr(y),
                                         _ptr(workspace), workspace.numel(), _stream_handle(stream)))
        return y

    def prefill_chunk_static(self, packed: PackedWeights, layer: int, kv: KVCache, x, y, stream=None):
        """prefill_chunk on the library's static workspace (no workspace argument, nothing allocated by the call)."""
        t = int(x.shape[0])
        _check(self.lib.rs_prefill_chunk_static(self.handle, C.byref(packed.struct), layer, kv.handle, _ptr(x), t, _ptr(y),
                                                _stream_handle(stream)))
        return y

    def static_workspace_bytes(self) -> int:
        return int(self.lib.rs_static_workspace_bytes())

    def prefill_batch(self, packed: PackedWeights, layer: int, kvs: Sequence[KVCache], chunk_lens: Sequence[int],
                      x, y, workspace, stream=None):
        """One micro-batch of several requests through one layer; x, y: bf16 [sum chunk_lens, H]."""
        r = len(kvs)
        arr_kv = (C.c_void_p * max(r, 1))(*[k.handle.value for k in kvs])
        arr_len = (C.c_int * max(r, 1))(*[int(n) for n in chunk_lens])
        _check(self.lib.rs_prefill_batch(self.handle, C.byref(packed.struct), layer, arr_kv, arr_len, r, _ptr(x), _ptr(y),
                                         _ptr(workspace), workspace.numel(), _stream_handle(stream)))
        return y

    def set_mrope_sections(self, temporal: int, height: int, width: int):
        _check(self.lib.rs_ctx_set_mrope_sections(self.handle, temporal, height, width))

    def prefill_batch_mrope(self, packed: PackedWeights, layer: int, kvs: Sequence[KVCache], chunk_lens: Sequence[int],
                            positions, x, y, workspace, stream=None):
        """rs_prefill_batch with explicit (temporal, height, width) rotary positions: positions is an int array-like
        [sum chunk_lens, 3] on the host."""
        r = len(kvs)
        flat = [int(v) for row in positions for v in row]
        arr_pos = (C.c_int * max(len(flat), 1))(*flat)
        arr_kv = (C.c_void_p * max(r, 1))(*[k.handle.value for k in kvs])
        arr_len = (C.c_int * max(r, 1))(*[int(n) for n in chunk_lens])
        _check(self.lib.rs_prefill_batch_mrope(self.handle, C.byref(packed.struct), layer, arr_kv, arr_len, r, arr_pos, _ptr(x),
                                               _ptr(y), _ptr(workspace), workspace.numel(), _stream_handle(stream)))
        return y

    def prefill_model_batch(self, layers: Sequence[PackedWeights], kvs: Sequence[KVCache], chunk_lens: Sequence[int],
                            x, y, workspace, stream=None):
        """One micro-batch through all stacked layers in one call; x, y: bf16 [sum chunk_lens, H]."""
        r = len(kvs)
        arr_w = (_Weights * max(len(layers), 1))(*[l.struct for l in layers])
        arr_kv = (C.c_void_p * max(r, 1))(*[k.handle.value for k in kvs])
        arr_len = (C.c_int * max(r, 1))(*[int(n) for n in chunk_lens])
        _check(self.lib.rs_prefill_model_batch(self.handle, arr_w, len(layers), arr_kv, arr_len, r, _ptr(x), _ptr(y),
                                               _ptr(workspace), workspace.numel(), _stream_handle(stream)))
        return y

    def prefill_model_batch_mrope(self, layers: Sequence[PackedWeights], kvs: Sequence[KVCache], chunk_lens: Sequence[int],
                                  positions, x, y, workspace, stream=None):
        """prefill_model_batch with explicit (temporal, height, width) rotary positions [sum chunk_lens, 3] (host)."""
        r = len(kvs)
        flat = [int(v) for row in positions for v in row]
        arr_pos = (C.c_int * max(len(flat), 1))(*flat)
        arr_w = (_Weights * max(len(layers), 1))(*[l.struct for l in layers])
        arr_kv = (C.c_void_p * max(r, 1))(*[k.handle.value for k in kvs])
        arr_len = (C.c_int * max(r, 1))(*[int(n) for n in chunk_lens])
        _check(self.lib.rs_prefill_model_batch_mrope(self.handle, arr_w, len(layers), arr_kv, arr_len, r, arr_pos, _ptr(x), _ptr(y),
                                                     _ptr(workspace), workspace.numel(), _stream_handle(stream)))
        return y

    def lm_head(self, final_norm_gain, w_lm, x_rows, stream=None):
        """fp32 logits [n_rows, vocab] of bf16 hidden-state rows x_rows [n_rows, H]: final RMSNorm + vocabulary projection."""
        import torch
        n, vocab = int(x_rows.shape[0]), int(w_lm.shape[0])
        logits = torch.empty((n, vocab), dtype=torch.float32, device=x_rows.device)
        ws = torch.empty(max(int(self.lib.rs_lm_head_workspace_bytes(self.handle, n)), 256), dtype=torch.uint8, device=x_rows.device)
        _check(self.lib.rs_lm_head(self.handle, _ptr(final_norm_gain), _ptr(w_lm), vocab, _ptr(x_rows), n, _ptr(logits),
                                   _ptr(ws), ws.numel(), _stream_handle(stream)))
        return logits


class Scheduler:
    """rs_sched: embedding tracker + Algorithm 1 encoder batching + Algorithm 2 token scheduling (host only)."""

    def __init__(self, token_budget: int):
        self._lib = load_library()
        h = C.c_void_p()
        _check(self._lib.rs_sched_create(int(token_budget), C.byref(h)))
        self._h = h

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib.rs_sched_destroy(self._h)
            self._h = None

    def add_request(self, request_id: int, segments: Sequence[Tuple[bool, int]]):
        arr = (_Segment * max(len(segments), 1))(*[_Segment(int(bool(m)), int(n)) for m, n in segments])
        _check(self._lib.rs_sched_add_request(self._h, request_id, arr, len(segments)))

    def mark_ready(self, request_id: int, segment: int):
        _check(self._lib.rs_sched_mark_ready(self._h, request_id, segment))

    def schedulable_tokens(self, request_id: int) -> int:
        return self._lib.rs_sched_schedulable_tokens(self._h, request_id)

    def prompt_length(self, request_id: int) -> int:
        return self._lib.rs_sched_prompt_length(self._h, request_id)

    def prefilled_tokens(self, request_id: int) -> int:
        return self._lib.rs_sched_prefilled_tokens(self._h, request_id)

    def encoder_batches(self, request_id: int, min_tokens: int, capacity: int = 4096) -> List[Tuple[int, int, int, int]]:
        out = (_EncodeBatch * max(capacity, 1))()
        n = C.c_int()
        _check(self._lib.rs_sched_encoder_batches(self._h, request_id, min_tokens, out, capacity, C.byref(n)))
        return [(b.first_segment, b.last_segment, b.n_items, b.n_tokens) for b in out[: n.value]]

    def next_round(self, capacity: Optional[int] = None) -> List[Tuple[int, int, int, bool]]:
        cap = self.queue_length() if capacity is None else capacity
        out = (_RoundEntry * max(cap, 1))()
        n = C.c_int()
        _check(self._lib.rs_sched_next_round(self._h, out, cap, C.byref(n)))
        return [(e.request_id, e.first_token, e.n_tokens, bool(e.finished)) for e in out[: n.value]]

    def queue_length(self) -> int:
        return self._lib.rs_sched_queue_length(self._h)

    def queue_ids(self) -> List[int]:
        cap = self.queue_length()
        out = (C.c_int64 * max(cap, 1))()
        n = C.c_int()
        _check(self._lib.rs_sched_queue_ids(self._h, out, cap, C.byref(n)))
        return list(out[: n.value])

    def release_request(self, request_id: int):
        _check(self._lib.rs_sched_release_request(self._h, request_id))
