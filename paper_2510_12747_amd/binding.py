"""ctypes binding of liblcsa.so: argument marshalling only.

Function names and argument order follow include/lcsa.h.  Tensors are torch CUDA
(ROCm) tensors used purely as device memory; every step of the path runs in the
library's own kernels.  There is no CPU fallback: if the shared library is missing
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch  # imported first so that the HIP runtime torch ships is the one the library binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblcsa.so")

LCSA_EVICT_SLIDING, LCSA_EVICT_IMPORTANCE_HEADWISE, LCSA_EVICT_IMPORTANCE_UNIFORM = 0, 1, 2
LCSA_F32, LCSA_BF16 = 0, 1
LCSA_BWD_AUTO, LCSA_BWD_FLOAT = 0, 1
WINDOW_TRUNCATED, WINDOW_PRESERVED = 0, 1


class LcsaError(RuntimeError):
    pass


class lcsa_geom(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "heads", "head_dim", "grid_h", "grid_w", "tile_h", "tile_w", "tile_t", "q_frames", "cache_frames",
        "radius_h", "radius_w", "window_mode", "topk", "dtype")]


@dataclass(frozen=True)
class Geom:
    heads: int
    head_dim: int
    grid_h: int
    grid_w: int
    tile_h: int
    tile_w: int
    q_frames: int
    cache_frames: int
    radius_h: int
    radius_w: int
    topk: int
    dtype: int = LCSA_BF16
    window_mode: int = WINDOW_TRUNCATED
    tile_t: int = 1          # frames per block; (tile_t, tile_h, tile_w) = (2, 8, 8) is the paper's partition

    def c(self) -> lcsa_geom:
        return lcsa_geom(self.heads, self.head_dim, self.grid_h, self.grid_w, self.tile_h, self.tile_w, self.tile_t,
                         self.q_frames, self.cache_frames, self.radius_h, self.radius_w, self.window_mode,
                         self.topk, self.dtype)

    @property
    def nb(self) -> int:
        return -(-self.grid_h // self.tile_h) * -(-self.grid_w // self.tile_w)

    @property
    def tokens_per_frame(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def n_qb(self) -> int:
        """Query blocks per chunk."""
        return self.q_frames // self.tile_t * self.nb

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == LCSA_BF16 else torch.float32


_lib = None
_vp, _i32, _i64, _f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
_gp = ctypes.POINTER(lcsa_geom)


def lib():
    """Loads liblcsa.so (built in-tree by paper_2510_12747_amd.build); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise LcsaError(f"{LIB_PATH} not found: build it with `python -m paper_2510_12747_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.lcsa_cache_device_bytes.restype = ctypes.c_size_t
        L.lcsa_cache_device_bytes.argtypes = [_gp]
        L.lcsa_cache_init.argtypes = [ctypes.POINTER(_vp), _gp, _vp, ctypes.c_size_t]
        L.lcsa_cache_reset.argtypes = [_vp]
        L.lcsa_cache_free.argtypes = [_vp]
        L.lcsa_cache_free.restype = None
        L.lcsa_cache_valid_frames.argtypes = [_vp]
        L.lcsa_cache_pooled_k_device.argtypes = [_vp]
        L.lcsa_cache_pooled_k_device.restype = _vp
        L.lcsa_cache_frame_slot.argtypes = [_vp, _i32]
        L.lcsa_kv_cache_append.argtypes = [_vp, _vp, _vp, _i64, _i64, _i32, _vp]
        L.lcsa_pool_blocks.argtypes = [_gp, _vp, _i64, _i64, _i32, _vp, _vp]
        L.lcsa_rope_pool_blocks.argtypes = [_gp, _vp, _i64, _i64, _i32, _i32, _i32, _i32, _f32, _i32, _vp, _i64, _i64, _vp, _vp]
        L.lcsa_select_blocks.argtypes = [_gp, _vp, _vp, _vp, _vp, _vp, _vp]
        L.lcsa_sparse_attn_fwd.argtypes = [_gp, _vp, _i64, _i64, _vp, _vp, _vp, _vp, _i64, _i64, _vp, _f32, _vp]
        L.lcsa_sparse_attn_bwd.argtypes = [_gp, _vp, _i64, _i64, _vp, _vp, _i64, _i64, _i32, _vp, _vp, _vp, _i64, _i64, _vp,
                                           _vp, _vp, _vp, _vp, _f32, _i32, _vp]
        L.lcsa_cache_v_clamped_device.argtypes = [_vp]
        L.lcsa_cache_v_clamped_device.restype = _vp
        L.lcsa_pool_select_blocks.argtypes = [_gp, _vp, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp]
        L.lcsa_cache_set_eviction.argtypes = [_vp, _i32]
        L.lcsa_cache_eviction.argtypes = [_vp]
        L.lcsa_block_importance.argtypes = [_gp, _vp, _vp, _f32, _vp]
        L.lcsa_block_importance_static.argtypes = [_gp, _vp, _vp, _f32, _vp]
        L.lcsa_cache_importance_device.argtypes = [_vp]
        L.lcsa_cache_importance_device.restype = _vp
        L.lcsa_cache_order_device.argtypes = [_vp]
        L.lcsa_cache_order_device.restype = _vp
        L.lcsa_status_string.restype = ctypes.c_char_p
        L.lcsa_status_string.argtypes = [_i32]
        L.lcsa_last_hip_error.restype = ctypes.c_char_p
        for f in ("lcsa_cache_init", "lcsa_cache_reset", "lcsa_cache_valid_frames", "lcsa_cache_frame_slot",
                  "lcsa_kv_cache_append", "lcsa_pool_blocks", "lcsa_select_blocks", "lcsa_sparse_attn_fwd",
                  "lcsa_pool_select_blocks", "lcsa_cache_set_eviction", "lcsa_cache_eviction", "lcsa_block_importance", "lcsa_sparse_attn_bwd", "lcsa_rope_pool_blocks",
                  "lcsa_block_importance_static"):
            getattr(L, f).restype = _i32
        _lib = L
    return _lib


def _check(status: int, what: str) -> None:
    if status != 0:
        L = lib()
        msg = L.lcsa_status_string(status).decode()
        if status == -3:
            msg += ": " + L.lcsa_last_hip_error().decode()
        raise LcsaError(f"{what}: {msg} ({status})")


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _tok(x: torch.Tensor):
    """[tokens][heads][d] device tensor -> (pointer, stride_tok, stride_head)."""
    if not x.is_cuda or x.dim() != 3 or x.stride(2) != 1:
        raise LcsaError("expected a device tensor [tokens][heads][d] with contiguous d")
    return x.data_ptr(), x.stride(0), x.stride(1)


def lcsa_status_string(status: int) -> str:
    return lib().lcsa_status_string(status).decode()


def lcsa_cache_device_bytes(geom: Geom) -> int:
    g = geom.c()
    return lib().lcsa_cache_device_bytes(ctypes.byref(g))


class Cache:
    """Host handle of one layer's sliding-window cache plus the torch buffer that backs it."""

    def __init__(self, geom: Geom, device="cuda:0"):
        n = lcsa_cache_device_bytes(geom)
        if n == 0:
            raise LcsaError("lcsa_cache_device_bytes: invalid geometry")
        self.geom = geom
        self.storage = torch.empty(n + 256, dtype=torch.uint8, device=device)
        self._base = (self.storage.data_ptr() + 255) // 256 * 256
        self.handle = _vp()
        g = geom.c()
        _check(lib().lcsa_cache_init(ctypes.byref(self.handle), ctypes.byref(g), _vp(self._base), n), "lcsa_cache_init")

    def __del__(self):
        if getattr(self, "handle", None):
            try:
                lib().lcsa_cache_free(self.handle)
            except Exception:      # interpreter shutdown: the module globals may already be gone
                pass
            self.handle = None


def lcsa_cache_init(geom: Geom, device="cuda:0") -> Cache:
    return Cache(geom, device)


def lcsa_cache_reset(cache: Cache) -> None:
    _check(lib().lcsa_cache_reset(cache.handle), "lcsa_cache_reset")


def lcsa_cache_valid_frames(cache: Cache) -> int:
    return lib().lcsa_cache_valid_frames(cache.handle)


def lcsa_cache_frame_slot(cache: Cache, frame: int) -> int:
    s = lib().lcsa_cache_frame_slot(cache.handle, frame)
    if s < 0:
        _check(s, "lcsa_cache_frame_slot")
    return s


def lcsa_cache_set_eviction(cache: Cache, policy: int) -> None:
    _check(lib().lcsa_cache_set_eviction(cache.handle, policy), "lcsa_cache_set_eviction")


def lcsa_cache_eviction(cache: Cache) -> int:
    return lib().lcsa_cache_eviction(cache.handle)


def lcsa_block_importance(geom: Geom, pooled_q: torch.Tensor, cache: Cache, scale: float = 0.0, stream=None) -> torch.Tensor:
    """Scores the visible groups for the next append; returns the view lcsa_cache_importance gives."""
    assert pooled_q.is_contiguous() and pooled_q.dtype == torch.float32
    assert pooled_q.shape == (geom.heads, geom.n_qb, geom.head_dim)
    g = geom.c()
    _check(lib().lcsa_block_importance(ctypes.byref(g), pooled_q.data_ptr(), cache.handle, scale, _stream(stream)),
           "lcsa_block_importance")
    return lcsa_cache_importance(cache)


def lcsa_block_importance_static(geom: Geom, pooled_q: torch.Tensor, cache: Cache, scale: float = 0.0, stream=None) -> torch.Tensor:
    """lcsa_block_importance with the library's static scratch array (allocates nothing)."""
    assert pooled_q.is_contiguous() and pooled_q.dtype == torch.float32
    assert pooled_q.shape == (geom.heads, geom.n_qb, geom.head_dim)
    g = geom.c()
    _check(lib().lcsa_block_importance_static(ctypes.byref(g), pooled_q.data_ptr(), cache.handle, scale, _stream(stream)),
           "lcsa_block_importance_static")
    return lcsa_cache_importance(cache)


def _cache_view(cache: Cache, ptr: int, dtype) -> torch.Tensor:
    g = cache.geom
    n = g.heads * (g.cache_frames // g.tile_t)
    off = ptr - cache.storage.data_ptr()
    return cache.storage[off:off + 4 * n].view(dtype).view(g.heads, g.cache_frames // g.tile_t)


def lcsa_cache_importance(cache: Cache) -> torch.Tensor:
    """float view [heads][cache_frames/tile_t] over the cache storage: importance by visible group (0 = oldest)."""
    return _cache_view(cache, lib().lcsa_cache_importance_device(cache.handle), torch.float32)


def lcsa_cache_order(cache: Cache) -> torch.Tensor | None:
    """int32 view [heads][cache_frames/tile_t]: visible group -> slot, per head; None under the sliding window."""
    ptr = lib().lcsa_cache_order_device(cache.handle)
    return _cache_view(cache, ptr, torch.int32) if ptr else None


def lcsa_cache_pooled_k(cache: Cache) -> torch.Tensor:
    """Pooled keys as a float tensor view [heads][(cache_frames/tile_t)*nb][d] over the cache storage (ring-slot order)."""
    g = cache.geom
    ptr = lib().lcsa_cache_pooled_k_device(cache.handle)
    off = ptr - cache.storage.data_ptr()
    rows = g.cache_frames // g.tile_t * g.nb
    n = g.heads * rows * g.head_dim
    return cache.storage[off:off + 4 * n].view(torch.float32).view(g.heads, rows, g.head_dim)


def lcsa_cache_v_clamped(cache: Cache) -> torch.Tensor:
    """int32 view [heads][(cache_frames/tile_t)*nb] over the cache storage (ring-slot order): values of V that the
    append clamped to half's range when it stored that block."""
    g = cache.geom
    ptr = lib().lcsa_cache_v_clamped_device(cache.handle)
    off = ptr - cache.storage.data_ptr()
    rows = g.cache_frames // g.tile_t * g.nb
    return cache.storage[off:off + 4 * g.heads * rows].view(torch.int32).view(g.heads, rows)


def lcsa_kv_cache_append(cache: Cache, k: torch.Tensor, v: torch.Tensor, n_frames: int, stream=None) -> None:
    kp, st, sh = _tok(k)
    vp, vst, vsh = _tok(v)
    if (st, sh) != (vst, vsh) or k.dtype != cache.geom.torch_dtype or v.dtype != k.dtype:
        raise LcsaError("lcsa_kv_cache_append: k and v must share strides and the cache dtype")
    if k.shape != (n_frames * cache.geom.tokens_per_frame, cache.geom.heads, cache.geom.head_dim) or v.shape != k.shape:
        raise LcsaError("lcsa_kv_cache_append: shape mismatch")
    _check(lib().lcsa_kv_cache_append(cache.handle, kp, vp, st, sh, n_frames, _stream(stream)), "lcsa_kv_cache_append")


def lcsa_pool_blocks(geom: Geom, x: torch.Tensor, n_frames: int, pooled: torch.Tensor | None = None, stream=None):
    xp, st, sh = _tok(x)
    if x.dtype != geom.torch_dtype or x.shape != (n_frames * geom.tokens_per_frame, geom.heads, geom.head_dim):
        raise LcsaError("lcsa_pool_blocks: shape/dtype mismatch")
    n_blocks = n_frames // geom.tile_t * geom.nb
    if pooled is None:
        pooled = torch.empty(geom.heads, n_blocks, geom.head_dim, dtype=torch.float32, device=x.device)
    assert pooled.is_contiguous() and pooled.dtype == torch.float32 and pooled.numel() == geom.heads * n_blocks * geom.head_dim
    g = geom.c()
    _check(lib().lcsa_pool_blocks(ctypes.byref(g), xp, st, sh, n_frames, pooled.data_ptr(), _stream(stream)), "lcsa_pool_blocks")
    return pooled


def lcsa_rope_pool_blocks(geom: Geom, x: torch.Tensor, n_frames: int, pairs, base: float = 0.0, first_frame: int = 0,
                          x_rot: torch.Tensor | None = None, pooled: torch.Tensor | None = None, stream=None):
    """Rotary embedding per (frame, row, column) axis + pooling in one pass; returns (x_rot, pooled).  x_rot may be x."""
    xp, st, sh = _tok(x)
    if x.dtype != geom.torch_dtype or x.shape != (n_frames * geom.tokens_per_frame, geom.heads, geom.head_dim):
        raise LcsaError("lcsa_rope_pool_blocks: shape/dtype mismatch")
    if x_rot is None:
        x_rot = torch.empty_like(x, memory_format=torch.contiguous_format)
    rp, rst, rsh = _tok(x_rot)
    assert x_rot.shape == x.shape and x_rot.dtype == x.dtype
    n_blocks = n_frames // geom.tile_t * geom.nb
    if pooled is None:
        pooled = torch.empty(geom.heads, n_blocks, geom.head_dim, dtype=torch.float32, device=x.device)
    assert pooled.is_contiguous() and pooled.dtype == torch.float32 and pooled.numel() == geom.heads * n_blocks * geom.head_dim
    g = geom.c()
    _check(lib().lcsa_rope_pool_blocks(ctypes.byref(g), xp, st, sh, n_frames, pairs[0], pairs[1], pairs[2], base, first_frame,
                                       rp, rst, rsh, pooled.data_ptr(), _stream(stream)), "lcsa_rope_pool_blocks")
    return x_rot, pooled


def lcsa_select_blocks(geom: Geom, pooled_q: torch.Tensor, cache: Cache, sel_idx=None, sel_cnt=None, gap=None,
                       want_gap: bool = True, stream=None):
    n_qb = geom.n_qb
    dev = pooled_q.device
    assert pooled_q.is_contiguous() and pooled_q.dtype == torch.float32 and pooled_q.shape == (geom.heads, n_qb, geom.head_dim)
    if sel_idx is None:
        sel_idx = torch.empty(geom.heads, n_qb, geom.topk, dtype=torch.int32, device=dev)
    if sel_cnt is None:
        sel_cnt = torch.empty(geom.heads, n_qb, dtype=torch.int32, device=dev)
    if gap is None and want_gap:
        gap = torch.empty(geom.heads, n_qb, dtype=torch.float32, device=dev)
    assert sel_idx.is_contiguous() and sel_cnt.is_contiguous() and sel_idx.dtype == torch.int32 and sel_cnt.dtype == torch.int32
    assert sel_idx.numel() == geom.heads * n_qb * geom.topk and sel_cnt.numel() == geom.heads * n_qb
    g = geom.c()
    _check(lib().lcsa_select_blocks(ctypes.byref(g), pooled_q.data_ptr(), cache.handle, sel_idx.data_ptr(),
                                    sel_cnt.data_ptr(), gap.data_ptr() if gap is not None else None,
                                    _stream(stream)), "lcsa_select_blocks")
    return sel_idx, sel_cnt, gap


def lcsa_pool_select_blocks(geom: Geom, q: torch.Tensor, cache: Cache, pooled_q=None, sel_idx=None, sel_cnt=None, gap=None,
                            want_gap: bool = True, stream=None):
    """lcsa_pool_blocks + lcsa_select_blocks in one launch; returns (pooled_q, sel_idx, sel_cnt, gap)."""
    n_qb = geom.n_qb
    qp, qst, qsh = _tok(q)
    if q.dtype != geom.torch_dtype or q.shape != (geom.q_frames * geom.tokens_per_frame, geom.heads, geom.head_dim):
        raise LcsaError("lcsa_pool_select_blocks: q shape/dtype mismatch")
    dev = q.device
    if pooled_q is None:
        pooled_q = torch.empty(geom.heads, n_qb, geom.head_dim, dtype=torch.float32, device=dev)
    if sel_idx is None:
        sel_idx = torch.empty(geom.heads, n_qb, geom.topk, dtype=torch.int32, device=dev)
    if sel_cnt is None:
        sel_cnt = torch.empty(geom.heads, n_qb, dtype=torch.int32, device=dev)
    if gap is None and want_gap:
        gap = torch.empty(geom.heads, n_qb, dtype=torch.float32, device=dev)
    assert pooled_q.is_contiguous() and pooled_q.dtype == torch.float32 and pooled_q.numel() == geom.heads * n_qb * geom.head_dim
    assert sel_idx.is_contiguous() and sel_cnt.is_contiguous() and sel_idx.dtype == torch.int32 and sel_cnt.dtype == torch.int32
    assert sel_idx.numel() == geom.heads * n_qb * geom.topk and sel_cnt.numel() == geom.heads * n_qb
    g = geom.c()
    _check(lib().lcsa_pool_select_blocks(ctypes.byref(g), qp, qst, qsh, cache.handle, pooled_q.data_ptr(), sel_idx.data_ptr(),
                                         sel_cnt.data_ptr(), gap.data_ptr() if gap is not None else None,
                                         _stream(stream)), "lcsa_pool_select_blocks")
    return pooled_q, sel_idx, sel_cnt, gap


def lcsa_sparse_attn_fwd(geom: Geom, q: torch.Tensor, cache: Cache, sel_idx: torch.Tensor, sel_cnt: torch.Tensor,
                         o: torch.Tensor | None = None, lse: torch.Tensor | None = None, scale: float = 0.0,
                         stream=None):
    qp, qst, qsh = _tok(q)
    if q.dtype != geom.torch_dtype or q.shape != (geom.q_frames * geom.tokens_per_frame, geom.heads, geom.head_dim):
        raise LcsaError("lcsa_sparse_attn_fwd: q shape/dtype mismatch")
    if o is None:
        o = torch.empty_like(q, memory_format=torch.contiguous_format)
    op, ost, osh = _tok(o)
    assert o.shape == q.shape and o.dtype == q.dtype
    assert sel_idx.is_contiguous() and sel_cnt.is_contiguous() and sel_idx.dtype == torch.int32 and sel_cnt.dtype == torch.int32
    assert sel_idx.numel() == geom.heads * geom.n_qb * geom.topk
    if lse is not None:
        assert lse.is_contiguous() and lse.dtype == torch.float32 and lse.shape == (q.shape[0], geom.heads)
    g = geom.c()
    _check(lib().lcsa_sparse_attn_fwd(ctypes.byref(g), qp, qst, qsh, cache.handle, sel_idx.data_ptr(), sel_cnt.data_ptr(),
                                      op, ost, osh, lse.data_ptr() if lse is not None else None, scale,
                                      _stream(stream)), "lcsa_sparse_attn_fwd")
    return o


def lcsa_sparse_attn_bwd(geom: Geom, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, kv_frames: int,
                         sel_idx: torch.Tensor, sel_cnt: torch.Tensor, d_o: torch.Tensor,
                         lse: torch.Tensor, scale: float = 0.0, float_path: bool = False, stream=None):
    """Gradients (d_q, d_k, d_v), float32 [tokens][heads][d], of the attention on the kept pairs, and delta [tokens][heads].
    float_path: float FMA kernels for every shape (LCSA_BWD_FLOAT) instead of the matrix cores where they apply."""
    qp, qst, qsh = _tok(q)
    kp, kst, ksh = _tok(k)
    vp, vst, vsh = _tok(v)
    gp, gst, gsh = _tok(d_o)
    if (kst, ksh) != (vst, vsh):
        raise LcsaError("lcsa_sparse_attn_bwd: k and v must share strides")
    n = geom.tokens_per_frame
    if q.shape != (geom.q_frames * n, geom.heads, geom.head_dim) or k.shape != (kv_frames * n, geom.heads, geom.head_dim) \
            or v.shape != k.shape or d_o.shape != q.shape:
        raise LcsaError("lcsa_sparse_attn_bwd: shape mismatch")
    if any(x.dtype != geom.torch_dtype for x in (q, k, v, d_o)):
        raise LcsaError("lcsa_sparse_attn_bwd: dtype mismatch")
    assert lse.is_contiguous() and lse.dtype == torch.float32 and lse.shape == (q.shape[0], geom.heads)
    assert sel_idx.is_contiguous() and sel_cnt.is_contiguous() and sel_idx.dtype == torch.int32 and sel_cnt.dtype == torch.int32
    d_q = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    d_k = torch.empty(k.shape, dtype=torch.float32, device=q.device)
    d_v = torch.empty(k.shape, dtype=torch.float32, device=q.device)
    delta = torch.empty(q.shape[0], geom.heads, dtype=torch.float32, device=q.device)
    g = geom.c()
    _check(lib().lcsa_sparse_attn_bwd(ctypes.byref(g), qp, qst, qsh, kp, vp, kst, ksh, kv_frames, sel_idx.data_ptr(),
                                      sel_cnt.data_ptr(), gp, gst, gsh, lse.data_ptr(), d_q.data_ptr(), d_k.data_ptr(),
                                      d_v.data_ptr(), delta.data_ptr(), scale, 1 if float_path else 0, _stream(stream)),
           "lcsa_sparse_attn_bwd")
    return d_q, d_k, d_v, delta
