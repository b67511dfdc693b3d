"""Thin ctypes binding of libmixattn.so: argument marshalling only.

Function names mirror include/mixattn.h.  torch supplies device memory and the
current stream; every step of the attention path runs inside the library's kernels.
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmixattn.so")
_lib = None

FULL, SLIDING = 0, 1
F32, BF16 = 0, 1
PARAM_CHUNK_KEYS, PARAM_PREFILL_SIMPLE, PARAM_PREFILL_WAVES, PARAM_PREFILL_HEADS = 0, 2, 3, 4
PARAM_BALANCED, PARAM_TEST_FAIL_ALLOC = 5, 6
ERR_SCRATCH = -10

EXPORTS = [
    "mixattn_validate_config", "mixattn_create_layout", "mixattn_create_layout_paged", "mixattn_destroy_layout",
    "mixattn_reset", "mixattn_release_sequence",
    "mixattn_append_kv", "mixattn_decode", "mixattn_decode_noalloc", "mixattn_append_decode",
    "mixattn_reserve_prefill", "mixattn_release_prefill", "mixattn_staging_bytes", "mixattn_reserve_steps", "mixattn_account_replays", "mixattn_decode_group", "mixattn_prefill", "mixattn_prefill_varlen",
    "mixattn_load_kv", "mixattn_n_caches",
    "mixattn_cache_of", "mixattn_seq_len", "mixattn_slot_of", "mixattn_slot_for", "mixattn_read_cache",
    "mixattn_read_device_lens", "mixattn_kv_bytes_allocated", "mixattn_kv_bytes_live", "mixattn_step_read_bytes",
    "mixattn_set_param", "mixattn_get_param", "mixattn_strerror", "mixattn_last_hip_error", "mixattn_version",
]


class MixAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load().mixattn_strerror(status).decode()
        super().__init__("%s: %s (status %d, hip error %d)" % (where, msg, status, load().mixattn_last_hip_error()))


class LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("window", C.c_int32), ("cache_id", C.c_int32)]


class Config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("layers", C.POINTER(LayerDesc)), ("batch", C.c_int32),
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("capacity", C.POINTER(C.c_int32)), ("kv_dtype", C.c_int32), ("out_dtype", C.c_int32),
        ("softmax_scale", C.c_float),
    ]


def load():
    """Loads libmixattn.so (built by __graft_entry__.build()); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libmixattn.so is not built: run `python __graft_entry__.py` (needs hipcc)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    lib.mixattn_validate_config.argtypes = [C.POINTER(Config)]
    lib.mixattn_create_layout.argtypes = [C.POINTER(Config), C.POINTER(vp)]
    lib.mixattn_create_layout_paged.argtypes = [C.POINTER(Config), i32, i64, C.POINTER(vp)]
    lib.mixattn_release_sequence.argtypes = [vp, i32, vp]
    lib.mixattn_destroy_layout.argtypes = [vp]
    lib.mixattn_reset.argtypes = [vp, vp]
    lib.mixattn_append_kv.argtypes = [vp, i32, vp, vp, vp]
    lib.mixattn_decode.argtypes = [vp, i32, vp, vp, vp]
    lib.mixattn_decode_noalloc.argtypes = [vp, i32, vp, vp, vp]
    lib.mixattn_reserve_prefill.argtypes = [vp, i32]
    lib.mixattn_release_prefill.argtypes = [vp]
    lib.mixattn_reserve_steps.argtypes = [vp, i32, vp]
    lib.mixattn_account_replays.argtypes = [vp, i32]
    lib.mixattn_append_decode.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.mixattn_decode_group.argtypes = [vp, C.POINTER(C.c_int32), i32, vp, vp, vp, vp, vp]
    lib.mixattn_prefill.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp]
    lib.mixattn_prefill_varlen.argtypes = [vp, i32, vp, vp, vp, vp, C.POINTER(C.c_int32), vp]
    lib.mixattn_load_kv.argtypes = [vp, i32, vp, vp, C.POINTER(C.c_int32), vp]
    lib.mixattn_n_caches.argtypes = [vp]
    lib.mixattn_cache_of.argtypes = [vp, i32, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.mixattn_seq_len.argtypes = [vp, i32, i32, C.POINTER(i64)]
    lib.mixattn_slot_of.argtypes = [vp, i32, i64, C.POINTER(i64)]
    lib.mixattn_slot_for.argtypes = [i32, i32, i64, C.POINTER(i64)]
    lib.mixattn_read_cache.argtypes = [vp, i32, i32, i32, i64, vp, vp]
    lib.mixattn_read_device_lens.argtypes = [vp, i32, C.POINTER(C.c_int32)]
    for f in ("mixattn_kv_bytes_allocated", "mixattn_kv_bytes_live", "mixattn_staging_bytes"):
        getattr(lib, f).argtypes = [vp]
        getattr(lib, f).restype = i64
    lib.mixattn_step_read_bytes.argtypes = [vp, i32]
    lib.mixattn_step_read_bytes.restype = i64
    lib.mixattn_set_param.argtypes = [vp, i32, i64]
    lib.mixattn_get_param.argtypes = [vp, i32, C.POINTER(i64)]
    lib.mixattn_strerror.argtypes = [i32]
    lib.mixattn_strerror.restype = C.c_char_p
    lib.mixattn_last_hip_error.argtypes = []
    lib.mixattn_version.argtypes = []
    lib.mixattn_version.restype = C.c_char_p
    _lib = lib
    return lib


def _dt(name) -> int:
    return {"f32": F32, "bf16": BF16, F32: F32, BF16: BF16}[name]


def make_config(layers: Sequence[Tuple[int, int, int]], batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                capacity: Optional[Sequence[int]], kv_dtype="bf16", out_dtype="f32", softmax_scale: float = 0.0):
    """Returns (Config, keepalive) for the C calls."""
    arr = (LayerDesc * max(1, len(layers)))()
    for i, (k, w, c) in enumerate(layers):
        arr[i].kind, arr[i].window, arr[i].cache_id = int(k), int(w), int(c)
    cap = None
    if capacity is not None:
        cap = (C.c_int32 * len(capacity))(*[int(x) for x in capacity])
    cfg = Config(len(layers), arr, batch, n_q_heads, n_kv_heads, head_dim,
                 cap if cap is not None else C.POINTER(C.c_int32)(), _dt(kv_dtype), _dt(out_dtype), softmax_scale)
    return cfg, (arr, cap)


def validate_config(*args, **kw) -> int:
    cfg, _keep = make_config(*args, **kw)
    return load().mixattn_validate_config(C.byref(cfg))


def slot_for(kind: int, window: int, pos: int) -> int:
    out = C.c_int64()
    st = load().mixattn_slot_for(kind, window, pos, C.byref(out))
    if st != 0:
        raise MixAttnError(st, "mixattn_slot_for")
    return out.value


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to mixattn must be contiguous device tensors")
    return t.data_ptr()


class Layout:
    """Owns one mixattn_layout handle.  Methods mirror the C entry points one to one."""

    def __init__(self, layers, batch, n_q_heads, n_kv_heads, head_dim, capacity=None, kv_dtype="bf16",
                 out_dtype="f32", softmax_scale: float = 0.0, page_tokens: int = 0, pool_tokens: int = 0):
        self.lib = load()
        self.layers = [tuple(int(x) for x in t) for t in layers]
        self.batch, self.Hq, self.Hkv, self.d = batch, n_q_heads, n_kv_heads, head_dim
        self.kv_dtype, self.out_dtype = _dt(kv_dtype), _dt(out_dtype)
        self.kv_torch = torch.float32 if self.kv_dtype == F32 else torch.bfloat16
        self.out_torch = torch.float32 if self.out_dtype == F32 else torch.bfloat16
        cfg, self._keep = make_config(self.layers, batch, n_q_heads, n_kv_heads, head_dim, capacity, kv_dtype,
                                      out_dtype, softmax_scale)
        h = C.c_void_p()
        if page_tokens:
            st = self.lib.mixattn_create_layout_paged(C.byref(cfg), int(page_tokens), int(pool_tokens), C.byref(h))
        else:
            st = self.lib.mixattn_create_layout(C.byref(cfg), C.byref(h))
        if st != 0:
            raise MixAttnError(st, "mixattn_create_layout")
        self.h = h

    # -- lifetime
    def close(self):
        if getattr(self, "h", None):
            self.lib.mixattn_destroy_layout(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int, where: str):
        if st != 0:
            raise MixAttnError(st, where)

    def _dtype_check(self, t: torch.Tensor, want: torch.dtype, shape):
        if t.dtype != want or tuple(t.shape) != tuple(shape):
            raise ValueError("expected %s %s, got %s %s" % (want, tuple(shape), t.dtype, tuple(t.shape)))

    # -- hot path
    def release_sequence(self, b: int):
        self._check(self.lib.mixattn_release_sequence(self.h, int(b), _stream()), "mixattn_release_sequence")

    def reset(self):
        self._check(self.lib.mixattn_reset(self.h, _stream()), "mixattn_reset")

    def append_kv(self, layer: int, k: torch.Tensor, v: torch.Tensor):
        self._dtype_check(k, self.kv_torch, (self.batch, self.Hkv, self.d))
        self._dtype_check(v, self.kv_torch, (self.batch, self.Hkv, self.d))
        self._check(self.lib.mixattn_append_kv(self.h, layer, _ptr(k), _ptr(v), _stream()), "mixattn_append_kv")

    def decode(self, layer: int, q: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        self._dtype_check(q, self.kv_torch, (self.batch, self.Hq, self.d))
        if out is None:
            out = torch.empty((self.batch, self.Hq, self.d), dtype=self.out_torch, device=q.device)
        else:
            self._dtype_check(out, self.out_torch, (self.batch, self.Hq, self.d))
        self._check(self.lib.mixattn_decode(self.h, layer, _ptr(q), _ptr(out), _stream()), "mixattn_decode")
        return out

    def decode_noalloc(self, layer: int, q: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
        self._dtype_check(q, self.kv_torch, (self.batch, self.Hq, self.d))
        self._dtype_check(out, self.out_torch, (self.batch, self.Hq, self.d))
        self._check(self.lib.mixattn_decode_noalloc(self.h, layer, _ptr(q), _ptr(out), _stream()),
                    "mixattn_decode_noalloc")
        return out

    def reserve_prefill(self, max_chunk_tokens: int):
        self._check(self.lib.mixattn_reserve_prefill(self.h, int(max_chunk_tokens)), "mixattn_reserve_prefill")

    def release_prefill(self):
        self._check(self.lib.mixattn_release_prefill(self.h), "mixattn_release_prefill")

    def staging_bytes(self) -> int:
        return self.lib.mixattn_staging_bytes(self.h)

    def reserve_steps(self, steps: int):
        self._check(self.lib.mixattn_reserve_steps(self.h, int(steps), _stream()), "mixattn_reserve_steps")

    def account_replays(self, steps: int):
        self._check(self.lib.mixattn_account_replays(self.h, int(steps)), "mixattn_account_replays")

    def append_decode(self, layer: int, k: torch.Tensor, v: torch.Tensor, q: torch.Tensor,
                      out: Optional[torch.Tensor] = None) -> torch.Tensor:
        self._dtype_check(k, self.kv_torch, (self.batch, self.Hkv, self.d))
        self._dtype_check(v, self.kv_torch, (self.batch, self.Hkv, self.d))
        self._dtype_check(q, self.kv_torch, (self.batch, self.Hq, self.d))
        if out is None:
            out = torch.empty((self.batch, self.Hq, self.d), dtype=self.out_torch, device=q.device)
        else:
            self._dtype_check(out, self.out_torch, (self.batch, self.Hq, self.d))
        self._check(self.lib.mixattn_append_decode(self.h, layer, _ptr(k), _ptr(v), _ptr(q), _ptr(out), _stream()),
                    "mixattn_append_decode")
        return out

    def decode_group(self, layers: Sequence[int], q: torch.Tensor, k: Optional[torch.Tensor] = None,
                     v: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        n = len(layers)
        self._dtype_check(q, self.kv_torch, (n, self.batch, self.Hq, self.d))
        for t in (k, v):
            if t is not None:
                self._dtype_check(t, self.kv_torch, (self.batch, self.Hkv, self.d))
        if out is None:
            out = torch.empty((n, self.batch, self.Hq, self.d), dtype=self.out_torch, device=q.device)
        else:
            self._dtype_check(out, self.out_torch, (n, self.batch, self.Hq, self.d))
        arr = (C.c_int32 * max(n, 1))(*[int(l) for l in layers])
        self._check(self.lib.mixattn_decode_group(self.h, arr, n, _ptr(k), _ptr(v), _ptr(q), _ptr(out), _stream()),
                    "mixattn_decode_group")
        return out

    def prefill(self, layer: int, q: torch.Tensor, k: Optional[torch.Tensor], v: Optional[torch.Tensor],
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
        B, S = q.shape[0], q.shape[1]
        self._dtype_check(q, self.kv_torch, (self.batch, S, self.Hq, self.d))
        for t in (k, v):
            if t is not None:
                self._dtype_check(t, self.kv_torch, (self.batch, S, self.Hkv, self.d))
        if out is None:
            out = torch.empty((B, S, self.Hq, self.d), dtype=self.out_torch, device=q.device)
        else:
            self._dtype_check(out, self.out_torch, (B, S, self.Hq, self.d))
        self._check(self.lib.mixattn_prefill(self.h, layer, _ptr(q), _ptr(k), _ptr(v), _ptr(out), S, _stream()),
                    "mixattn_prefill")
        return out

    def prefill_varlen(self, layer: int, q: torch.Tensor, k: Optional[torch.Tensor], v: Optional[torch.Tensor],
                       seq_lens: Sequence[int], out: Optional[torch.Tensor] = None) -> torch.Tensor:
        total = int(sum(seq_lens))
        self._dtype_check(q, self.kv_torch, (total, self.Hq, self.d))
        for t in (k, v):
            if t is not None:
                self._dtype_check(t, self.kv_torch, (total, self.Hkv, self.d))
        if out is None:
            out = torch.empty((total, self.Hq, self.d), dtype=self.out_torch, device=q.device)
        else:
            self._dtype_check(out, self.out_torch, (total, self.Hq, self.d))
        if len(seq_lens) != self.batch:
            raise ValueError("seq_lens needs one entry per sequence")
        lens = (C.c_int32 * self.batch)(*[int(x) for x in seq_lens])
        self._check(self.lib.mixattn_prefill_varlen(self.h, layer, _ptr(q), _ptr(k), _ptr(v), _ptr(out), lens,
                                                    _stream()), "mixattn_prefill_varlen")
        return out

    def load_kv(self, layer: int, k: torch.Tensor, v: torch.Tensor, seq_lens: Sequence[int]):
        total = int(sum(seq_lens))
        self._dtype_check(k, self.kv_torch, (total, self.Hkv, self.d))
        self._dtype_check(v, self.kv_torch, (total, self.Hkv, self.d))
        lens = (C.c_int32 * self.batch)(*[int(x) for x in seq_lens])
        self._check(self.lib.mixattn_load_kv(self.h, layer, _ptr(k), _ptr(v), lens, _stream()), "mixattn_load_kv")

    # -- introspection
    def n_caches(self) -> int:
        return self.lib.mixattn_n_caches(self.h)

    def cache_of(self, layer: int) -> Tuple[int, bool]:
        ci, w = C.c_int(), C.c_int()
        self._check(self.lib.mixattn_cache_of(self.h, layer, C.byref(ci), C.byref(w)), "mixattn_cache_of")
        return ci.value, bool(w.value)

    def writer_of(self, layer: int) -> int:
        ci, _ = self.cache_of(layer)
        for li in range(len(self.layers)):
            c2, w2 = self.cache_of(li)
            if c2 == ci and w2:
                return li
        raise AssertionError("cache without writer")

    def seq_len(self, cache_index: int, b: int) -> int:
        n = C.c_int64()
        self._check(self.lib.mixattn_seq_len(self.h, cache_index, b, C.byref(n)), "mixattn_seq_len")
        return n.value

    def slot_of(self, cache_index: int, pos: int) -> int:
        s = C.c_int64()
        self._check(self.lib.mixattn_slot_of(self.h, cache_index, pos, C.byref(s)), "mixattn_slot_of")
        return s.value

    def read_cache(self, cache_index: int, b: int, kv_head: int, slot: int):
        """(k_row, v_row) as CPU tensors of kv_dtype."""
        k = torch.empty(self.d, dtype=self.kv_torch)
        v = torch.empty(self.d, dtype=self.kv_torch)
        self._check(self.lib.mixattn_read_cache(self.h, cache_index, b, kv_head, slot, k.data_ptr(), v.data_ptr()),
                    "mixattn_read_cache")
        return k, v

    def device_lens(self, cache_index: int) -> List[int]:
        arr = (C.c_int32 * self.batch)()
        self._check(self.lib.mixattn_read_device_lens(self.h, cache_index, arr), "mixattn_read_device_lens")
        return list(arr)

    def kv_bytes_allocated(self) -> int:
        return self.lib.mixattn_kv_bytes_allocated(self.h)

    def kv_bytes_live(self) -> int:
        return self.lib.mixattn_kv_bytes_live(self.h)

    def step_read_bytes(self, layer: int) -> int:
        return self.lib.mixattn_step_read_bytes(self.h, layer)

    def set_param(self, param: int, value: int):
        self._check(self.lib.mixattn_set_param(self.h, param, value), "mixattn_set_param")

    def get_param(self, param: int) -> int:
        v = C.c_int64()
        self._check(self.lib.mixattn_get_param(self.h, param, C.byref(v)), "mixattn_get_param")
        return v.value
