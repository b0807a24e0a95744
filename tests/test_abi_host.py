"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and
validates arguments on the host before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2510_12747_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lcsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lcsa_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    L = B.lib()
    names = declared_symbols()
    assert {"lcsa_pool_blocks", "lcsa_select_blocks", "lcsa_sparse_attn_fwd", "lcsa_kv_cache_append"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    assert B.lcsa_status_string(0) == "ok"
    assert "invalid" in B.lcsa_status_string(-1)
    assert "unsupported" in B.lcsa_status_string(-2)
    assert "HIP" in B.lcsa_status_string(-3)


PAPER = dict(heads=12, head_dim=128, grid_h=48, grid_w=88, tile_h=8, tile_w=16, q_frames=2, cache_frames=6,
             radius_h=24, radius_w=24, topk=32)


def up256(n):
    return -(-n // 256) * 256


def eviction_state_bytes(heads, groups, n_qb, nb):
    """visible-group -> slot table, importance per group, per-row scratch of the importance kernel, the ring
    words of the sliding window, clamped-V counts per tile"""
    return up256(heads * groups * 4) + up256(heads * groups * 4) + up256(heads * n_qb * groups * 4) + 256 \
        + up256(heads * groups * nb * 4)


def test_cache_bytes_formula():
    g = B.Geom(**PAPER)
    nb = 6 * 6
    tiles = 12 * 6 * nb
    assert g.nb == nb
    assert B.lcsa_cache_device_bytes(g) == 2 * tiles * 128 * 128 * 2 + tiles * 128 * 4 + eviction_state_bytes(12, 6, 72, 36)
    tiny = B.Geom(1, 32, 6, 8, 4, 4, 2, 4, 4, 4, 4, dtype=B.LCSA_F32)
    assert B.lcsa_cache_device_bytes(tiny) == 2 * (16 * 16 * 32 * 4) + 16 * 32 * 4 + eviction_state_bytes(1, 4, 8, 4)
    # (2,8,8) blocks on the paper grid: 66 blocks per frame pair, 3 pairs in the ring, 128 tokens per block
    paper288 = B.Geom(**{**PAPER, "tile_w": 8, "tile_t": 2})
    assert paper288.nb == 66 and paper288.n_qb == 66
    assert B.lcsa_cache_device_bytes(paper288) == 2 * (12 * 3 * 66) * 128 * 128 * 2 + (12 * 3 * 66) * 128 * 4 \
        + eviction_state_bytes(12, 3, 66, 66)


@pytest.mark.parametrize("field,value", [
    ("heads", 0), ("head_dim", 0), ("head_dim", 12), ("head_dim", 264), ("grid_h", 0), ("tile_w", 0),
    ("q_frames", 0), ("cache_frames", 1), ("topk", 0), ("dtype", 2), ("window_mode", 3), ("tile_t", 0), ("tile_t", 4),
])
def test_invalid_geometry_is_rejected(field, value):
    g = B.Geom(**{**PAPER, field: value})
    assert B.lcsa_cache_device_bytes(g) == 0
    L = B.lib()
    gc = g.c()
    h = ctypes.c_void_p()
    assert L.lcsa_cache_init(ctypes.byref(h), ctypes.byref(gc), ctypes.c_void_p(256), 1 << 40) == -1
    assert L.lcsa_pool_blocks(ctypes.byref(gc), 256, 1536, 128, 1, 256, None) == -1


def test_host_side_validation_without_gpu():
    """Every failing call below returns before any HIP call, so it runs on a GPU-less host."""
    L = B.lib()
    g = B.Geom(**PAPER)
    gc = g.c()
    n = B.lcsa_cache_device_bytes(g)
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(1 << 20)   # never dereferenced on the host
    assert L.lcsa_cache_init(ctypes.byref(h), ctypes.byref(gc), fake, n - 1) == -1          # too small
    assert L.lcsa_cache_init(ctypes.byref(h), ctypes.byref(gc), ctypes.c_void_p((1 << 20) + 16), n) == -1  # misaligned
    assert L.lcsa_cache_init(ctypes.byref(h), ctypes.byref(gc), None, n) == -1
    assert L.lcsa_cache_init(None, ctypes.byref(gc), fake, n) == -1
    assert L.lcsa_cache_init(ctypes.byref(h), ctypes.byref(gc), fake, n) == 0
    assert L.lcsa_cache_valid_frames(h) == 0
    assert L.lcsa_cache_frame_slot(h, 0) == -1
    # append: bad frame counts, null / misaligned pointers, short strides
    assert L.lcsa_kv_cache_append(h, fake, fake, 1536, 128, 0, None) == -1
    assert L.lcsa_kv_cache_append(h, fake, fake, 1536, 128, 7, None) == -1
    assert L.lcsa_kv_cache_append(h, None, fake, 1536, 128, 2, None) == -1
    assert L.lcsa_kv_cache_append(h, ctypes.c_void_p((1 << 20) + 2), fake, 1536, 128, 2, None) == -1
    assert L.lcsa_kv_cache_append(h, fake, fake, 64, 128, 2, None) == -1
    assert L.lcsa_kv_cache_append(h, fake, fake, 1540, 128, 2, None) == -1
    assert L.lcsa_kv_cache_append(None, fake, fake, 1536, 128, 2, None) == -1
    # select / attention on an empty cache
    assert L.lcsa_select_blocks(ctypes.byref(gc), fake, h, fake, fake, None, None) == -1
    assert L.lcsa_sparse_attn_fwd(ctypes.byref(gc), fake, 1536, 128, h, fake, fake, fake, 1536, 128, None, 0.0, None) == -1
    # geometry that disagrees with the cache's
    other = B.Geom(**{**PAPER, "grid_w": 80}).c()
    assert L.lcsa_select_blocks(ctypes.byref(other), fake, h, fake, fake, None, None) == -1
    assert L.lcsa_select_blocks(ctypes.byref(gc), None, h, fake, fake, None, None) == -1
    assert L.lcsa_pool_select_blocks(ctypes.byref(gc), fake, 1536, 128, h, fake, fake, fake, None, None) == -1   # empty cache
    assert L.lcsa_pool_select_blocks(ctypes.byref(gc), fake, 1536, 128, None, fake, fake, fake, None, None) == -1
    assert L.lcsa_pool_select_blocks(ctypes.byref(gc), fake, 64, 128, h, fake, fake, fake, None, None) == -1
    # eviction policy: host-only switch, valid values only, importance needs a non-empty cache
    assert L.lcsa_cache_eviction(h) == B.LCSA_EVICT_SLIDING and L.lcsa_cache_order_device(h) is None
    assert L.lcsa_cache_set_eviction(h, 3) == -1 and L.lcsa_cache_set_eviction(h, -1) == -1
    assert L.lcsa_cache_set_eviction(None, 1) == -1
    assert L.lcsa_cache_set_eviction(h, B.LCSA_EVICT_IMPORTANCE_UNIFORM) == 0
    assert L.lcsa_cache_eviction(h) == B.LCSA_EVICT_IMPORTANCE_UNIFORM and L.lcsa_cache_order_device(h) is not None
    assert L.lcsa_cache_frame_slot(h, 0) == -1
    assert L.lcsa_block_importance(ctypes.byref(gc), fake, h, 0.0, None) == -1      # nothing cached yet
    assert L.lcsa_block_importance(ctypes.byref(gc), None, h, 0.0, None) == -1
    assert L.lcsa_cache_set_eviction(h, B.LCSA_EVICT_SLIDING) == 0 and L.lcsa_cache_order_device(h) is None
    # more than 64 groups of capacity: importance policies are not built for that
    big = B.Geom(**{**PAPER, "grid_h": 8, "grid_w": 16, "cache_frames": 130}).c()
    hb = ctypes.c_void_p()
    assert L.lcsa_cache_init(ctypes.byref(hb), ctypes.byref(big), fake, 1 << 40) == 0
    assert L.lcsa_cache_set_eviction(hb, B.LCSA_EVICT_IMPORTANCE_HEADWISE) == -2
    L.lcsa_cache_free(hb)
    # backward: null pointers, too few key frames, short strides (no cache involved)
    L.lcsa_sparse_attn_bwd.restype = ctypes.c_int32
    bwd = lambda kvf=6, q=fake, dq=fake, st=1536: L.lcsa_sparse_attn_bwd(
        ctypes.byref(gc), q, st, 128, fake, fake, 1536, 128, kvf, fake, fake, fake, 1536, 128, fake, dq, fake, fake, fake,
        ctypes.c_float(0.0), 0, None)
    assert bwd(kvf=1) == -1 and bwd(q=None) == -1 and bwd(dq=None) == -1 and bwd(st=64) == -1
    big_block = B.Geom(**{**PAPER, "tile_h": 16, "tile_w": 32, "head_dim": 256}).c()      # 512 tokens x 256 channels per block
    assert L.lcsa_sparse_attn_bwd(ctypes.byref(big_block), fake, 3072, 256, fake, fake, 3072, 256, 6, fake, fake, fake, 3072, 256,
                                  fake, fake, fake, fake, fake, ctypes.c_float(0.0), 0, None) == -2
    assert L.lcsa_sparse_attn_bwd(ctypes.byref(gc), fake, 1536, 128, fake, fake, 1536, 128, 6, fake, fake, fake, 1536, 128, fake,
                                  fake, fake, fake, fake, ctypes.c_float(0.0), 7, None) == -1      # unknown arithmetic
    assert L.lcsa_cache_v_clamped_device(h) is not None
    assert L.lcsa_cache_reset(h) == 0
    assert L.lcsa_cache_reset(None) == -1
    assert L.lcsa_cache_valid_frames(None) == -1
    L.lcsa_cache_free(h)
    L.lcsa_cache_free(None)
