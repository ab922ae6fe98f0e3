"""Thin ctypes binding over the C ABI of include/hack.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
libhack_mi355x.so.  PyTorch is used for device memory and the current stream.
There is no CPU fallback: if the library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhack_mi355x.so")

HACK_BF16, HACK_F32 = 0, 1
CONTEXTUAL, STRUCTURAL = 0, 1

EXPORTS = [
    "hack_create", "hack_destroy", "hack_strerror", "hack_last_error", "hack_check",
    "hack_score", "hack_select", "hack_compact", "hack_attn", "hack_attn_variant",
    "hack_kvcache_rows_required", "hack_kvcache_create", "hack_kvcache_destroy",
    "hack_kvcache_reset", "hack_kvcache_view", "hack_step", "hack_head_variance",
    "hack_set_score_mode", "hack_get_score_mode", "hack_score_static", "hack_merge", "hack_step_final",
]


class HackError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"hack status {status}: {msg}")
        self.status = status


class hack_config(C.Structure):
    _fields_ = [("device", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32), ("dtype", C.c_int32),
                ("max_units", C.c_int32), ("max_cache_len", C.c_int32), ("max_queries", C.c_int32),
                ("n_obs", C.c_int32)]


class hack_cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("pos", C.c_void_p), ("rows", C.c_int64),
                ("off", C.POINTER(C.c_int64)), ("len", C.POINTER(C.c_int32))]


_lib = None


def load_library() -> C.CDLL:
    """dlopen the in-tree library; torch is imported first so that both use the
    same HIP runtime."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (loads libamdhip64 with the soname the library needs)
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2504_09261_amd.build` "
            "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    pi32, pi64, pu8 = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
    pcache = C.POINTER(hack_cache)
    lib.hack_create.argtypes = [C.POINTER(vp), C.POINTER(hack_config)]
    lib.hack_destroy.argtypes = [vp]
    lib.hack_destroy.restype = None
    lib.hack_strerror.argtypes = [C.c_int]
    lib.hack_strerror.restype = C.c_char_p
    lib.hack_last_error.argtypes = [vp]
    lib.hack_last_error.restype = C.c_char_p
    lib.hack_check.argtypes = [vp]
    lib.hack_set_score_mode.argtypes = [vp, i32]
    lib.hack_get_score_mode.argtypes = [vp]
    lib.hack_get_score_mode.restype = i32
    lib.hack_score.argtypes = [vp, i32, i32, vp, pi32, i32, f32, pcache, vp, pu8, vp, i64, vp]
    lib.hack_score_static.argtypes = [vp, i32, i32, vp, pi32, i32, f32, pcache, vp, pu8, vp, i64, vp]
    lib.hack_select.argtypes = [vp, i32, vp, i64, pi32, pu8, pi32, i32, i32, vp, i64, pi32, vp]
    lib.hack_compact.argtypes = [vp, i32, i32, pcache, vp, vp, i32, vp, i64, pcache, vp]
    lib.hack_merge.argtypes = [vp, i32, i32, pcache, vp, vp, vp, i64, pu8, pcache, vp]
    lib.hack_step_final.argtypes = [vp, vp, i32, i32, vp, vp, vp, pu8, pi32, i32, f32, vp, vp, i64, vp]
    lib.hack_attn.argtypes = [vp, i32, i32, vp, pcache, f32, vp, vp]
    lib.hack_attn_variant.argtypes = [vp, i32, i32]
    lib.hack_attn_variant.restype = i32
    lib.hack_head_variance.argtypes = [vp, i32, i32, vp, pcache, f32, vp, vp]
    lib.hack_kvcache_rows_required.argtypes = [i32, pi32, pi64]
    lib.hack_kvcache_create.argtypes = [vp, i32, pi32, vp, vp, vp, i64, C.POINTER(vp)]
    lib.hack_kvcache_destroy.argtypes = [vp]
    lib.hack_kvcache_destroy.restype = None
    lib.hack_kvcache_reset.argtypes = [vp]
    lib.hack_kvcache_view.argtypes = [vp, pcache]
    lib.hack_step.argtypes = [vp, vp, i32, i32, vp, vp, vp, pu8, pi32, i32, f32, vp, vp, i64, vp]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.restype is C.c_int and name not in ("hack_strerror", "hack_last_error"):
            fn.restype = C.c_int
    _lib = lib
    return lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint8)


def _p(a: Optional[np.ndarray], ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def _dev(t) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA/HIP tensors"
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


class Cache:
    """A hack_cache view: device K/V(/pos) tensors plus host offsets and lengths."""

    def __init__(self, k, v, off, length, pos=None):
        self.k, self.v, self.pos = k, v, pos
        self.off, self.len = _i64(off), _i32(length)
        assert k.shape == v.shape and k.dim() == 2
        self.rows = int(k.shape[0])

    def struct(self) -> hack_cache:
        return hack_cache(_dev(self.k), _dev(self.v), _dev(self.pos), self.rows,
                          _p(self.off, C.c_int64), _p(self.len, C.c_int32))


class ManagedCache:
    """hack_kvcache: two slabs of cap[u] rows per unit inside caller-provided tensors."""

    def __init__(self, hack: "Hack", cap: Sequence[int], with_pos: bool = True):
        import torch
        self.hack = hack
        self.cap = _i32(cap)
        lib = hack.lib
        rows = C.c_int64()
        hack._check(lib.hack_kvcache_rows_required(len(self.cap), _p(self.cap, C.c_int32), C.byref(rows)))
        self.rows = rows.value
        dev = torch.device("cuda", hack.device)
        self.k = torch.empty((self.rows, hack.head_dim), dtype=hack.torch_dtype, device=dev)
        self.v = torch.empty((self.rows, hack.head_dim), dtype=hack.torch_dtype, device=dev)
        self.pos = torch.empty((self.rows,), dtype=torch.int32, device=dev) if with_pos else None
        h = C.c_void_p()
        hack._check(lib.hack_kvcache_create(hack.ctx, len(self.cap), _p(self.cap, C.c_int32), _dev(self.k),
                                            _dev(self.v), _dev(self.pos), self.rows, C.byref(h)))
        self.handle = h

    def reset(self):
        self.hack._check(self.hack.lib.hack_kvcache_reset(self.handle))

    def view(self):
        """(off int64[U], len int32[U]) copies of the current state."""
        s = hack_cache()
        self.hack._check(self.hack.lib.hack_kvcache_view(self.handle, C.byref(s)))
        n = len(self.cap)
        return np.ctypeslib.as_array(s.off, (n,)).copy(), np.ctypeslib.as_array(s.len, (n,)).copy()

    def as_cache(self) -> Cache:
        off, ln = self.view()
        return Cache(self.k, self.v, off, ln, self.pos)

    def close(self):
        if self.handle:
            self.hack.lib.hack_kvcache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Hack:
    """One library context (one element type / head_dim, one stream at a time)."""

    def __init__(self, heads: int, head_dim: int, dtype: str, max_units: int, max_cache_len: int,
                 max_queries: int, n_obs: int = 32, device: int = 0):
        import torch
        self.lib = load_library()
        self.heads, self.head_dim, self.device = heads, head_dim, device
        self.dtype = dtype
        self.torch_dtype = torch.float32 if dtype == "f32" else torch.bfloat16
        cfg = hack_config(device, heads, head_dim, HACK_F32 if dtype == "f32" else HACK_BF16, max_units,
                          max_cache_len, max_queries, n_obs)
        ctx = C.c_void_p()
        st = self.lib.hack_create(C.byref(ctx), C.byref(cfg))
        if st != 0:
            raise HackError(st, self.lib.hack_strerror(st).decode())
        self.ctx = ctx

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.hack_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != 0:
            raise HackError(st, f"{self.lib.hack_strerror(st).decode()}: {self.lib.hack_last_error(self.ctx).decode()}")

    def check(self):
        """Raise if a kernel of an earlier call reported a problem (synchronise first)."""
        self._check(self.lib.hack_check(self.ctx))

    def set_score_mode(self, mode: int):
        """0: fused single launch (default); 1: two launches without in-kernel waits."""
        self._check(self.lib.hack_set_score_mode(self.ctx, mode))

    def score_mode(self) -> int:
        return int(self.lib.hack_get_score_mode(self.ctx))

    # ---- a1 ----
    def score(self, q, cache: Cache, scale: float, importance, k_new=None, q_idx=None, n_obs: Optional[int] = None,
              active=None):
        B, H, Nk, d = q.shape
        n_obs = min(32, Nk) if n_obs is None else n_obs
        qi = None if q_idx is None else _i32(q_idx)
        act = None if active is None else _u8(active)
        cs = cache.struct()
        self._check(self.lib.hack_score(self.ctx, B, Nk, _dev(q), _p(qi, C.c_int32), n_obs, scale, C.byref(cs),
                                        _dev(k_new), _p(act, C.c_uint8), _dev(importance),
                                        importance.stride(0), _stream()))

    def score_static(self, q, cache: Cache, scale: float, importance, k_new=None, q_idx=None,
                     n_obs: Optional[int] = None, active=None):
        """hack_score with all kernel scratch in the library's fixed device array (allocates nothing)."""
        B, H, Nk, d = q.shape
        n_obs = min(32, Nk) if n_obs is None else n_obs
        qi = None if q_idx is None else _i32(q_idx)
        act = None if active is None else _u8(active)
        cs = cache.struct()
        self._check(self.lib.hack_score_static(self.ctx, B, Nk, _dev(q), _p(qi, C.c_int32), n_obs, scale, C.byref(cs),
                                               _dev(k_new), _p(act, C.c_uint8), _dev(importance),
                                               importance.stride(0), _stream()))

    # ---- a2 ----
    def select(self, B: int, importance, t_in, head_type, budget, n_init: int, n_recent: int, kept_idx) -> np.ndarray:
        t_in, budget, ht = _i32(t_in), _i32(budget), _u8(head_type)
        len_out = np.zeros(len(t_in), np.int32)
        self._check(self.lib.hack_select(self.ctx, B, _dev(importance), importance.stride(0), _p(t_in, C.c_int32),
                                         _p(ht, C.c_uint8), _p(budget, C.c_int32), n_init, n_recent,
                                         _dev(kept_idx), kept_idx.stride(0), _p(len_out, C.c_int32), _stream()))
        return len_out

    # ---- a3 ----
    def compact(self, B: int, Nk: int, cache_in: Cache, kept_idx, cache_out: Cache, k_new=None, v_new=None,
                pos_new: int = 0):
        ci, co = cache_in.struct(), cache_out.struct()
        self._check(self.lib.hack_compact(self.ctx, B, Nk, C.byref(ci), _dev(k_new), _dev(v_new), pos_new,
                                          _dev(kept_idx), kept_idx.stride(0), C.byref(co), _stream()))

    def merge(self, B: int, Nk: int, cache_in: Cache, kept_idx, cache_out: Cache, k_new=None, v_new=None, active=None):
        """Final-step merge: evicted rows folded into their nearest kept rows of cache_out (in place)."""
        ci, co = cache_in.struct(), cache_out.struct()
        act = None if active is None else _u8(active)
        self._check(self.lib.hack_merge(self.ctx, B, Nk, C.byref(ci), _dev(k_new), _dev(v_new), _dev(kept_idx),
                                        kept_idx.stride(0), _p(act, C.c_uint8), C.byref(co), _stream()))

    # ---- a4 ----
    def attn(self, q, cache: Cache, scale: float, out):
        B, H, Nk, d = q.shape
        cs = cache.struct()
        self._check(self.lib.hack_attn(self.ctx, B, Nk, _dev(q), C.byref(cs), scale, _dev(out), _stream()))

    def attn_variant(self, B: int, N_k: int) -> int:
        """0: 128-query work items; 1: 32-query work items with the keys split over the waves."""
        v = int(self.lib.hack_attn_variant(self.ctx, B, N_k))
        if v < 0:
            self._check(v)
        return v

    # ---- offline head classification ----
    def head_variance(self, q, cache: Cache, scale: float, sigma):
        """sigma (device float64 [B*H]) <- sum of column variances of Softmax(scale q k^T) per unit."""
        B, H, Nk, d = q.shape
        cs = cache.struct()
        self._check(self.lib.hack_head_variance(self.ctx, B, Nk, _dev(q), C.byref(cs), scale, _dev(sigma), _stream()))

    # ---- a5 ----
    def managed_cache(self, cap, with_pos: bool = True) -> ManagedCache:
        return ManagedCache(self, cap, with_pos)

    def step(self, cache: ManagedCache, q, k_new, v_new, head_type, budget, n_init: int, scale: float, out,
             kept_idx=None, final: bool = False):
        """final=True: hack_step_final (the last scale step; contextual units merge what they discard)."""
        B, H, Nk, d = q.shape
        ht, bud = _u8(head_type), _i32(budget)
        fn = self.lib.hack_step_final if final else self.lib.hack_step
        self._check(fn(self.ctx, cache.handle, B, Nk, _dev(q), _dev(k_new), _dev(v_new),
                                       _p(ht, C.c_uint8), _p(bud, C.c_int32), n_init, scale, _dev(out),
                                       _dev(kept_idx), 0 if kept_idx is None else kept_idx.stride(0), _stream()))
