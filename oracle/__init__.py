"""CPU oracle for locality-constrained block-sparse attention -- TEST INFRASTRUCTURE.

Thin ctypes wrappers over ``lcsa_oracle.c`` (fp64, plain loops) plus a
list-based model of the sliding-window KV cache.  Only tests, the smoke check
and the benchmark's ``cpu_baseline`` leg may import this package; it shares no
code with the HIP library and never calls it.

Paper passages followed: Sec. 3.2 "Stage 2" (blocks, pooling, coarse map,
top-k, full attention on kept pairs), Sec. 3.3 / Fig. 3 (local window),
eq. (1) (softmax with 1/sqrt(d)), appendix "Discussion on Stream VSR
Pipelines" (sliding-window cache of recent latents + current chunk),
appendix on KV-cache eviction (importance-based eviction, head-wise and
uniform; the paper prints no numbers for it that could pin these functions:
their agreement with the authors' variant is unpinned).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lcsa_oracle.c")
_LIB_PATH = os.path.join(_HERE, "liblcsa_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile lcsa_oracle.c with gcc (OpenMP, -O2, no fast-math)."""
    stale = (not os.path.exists(_LIB_PATH)
             or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC))
    if force or stale:
        subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                        "-o", _LIB_PATH, _SRC, "-lm"], check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.lcsa_oracle_blocks_per_frame.restype = ctypes.c_int
        _lib.lcsa_oracle_allowed.restype = ctypes.c_int
        _lib.lcsa_oracle_threads.restype = ctypes.c_int
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


_f32, _f64, _i32 = ctypes.c_float, ctypes.c_double, ctypes.c_int32
_ci, _cl = ctypes.c_int, ctypes.c_int64


@dataclass(frozen=True)
class Geometry:
    """Problem geometry in the paper's terms (one block = tile_t frames x one th x tw tile)."""
    heads: int
    head_dim: int
    grid_h: int
    grid_w: int
    tile_h: int
    tile_w: int
    q_frames: int
    radius_h: int      # tokens between block centres; < 0: unbounded
    radius_w: int
    topk: int
    window_mode: int = 0   # 0 boundary-truncated, 1 boundary-preserved
    tile_t: int = 1        # frames per block; the paper's blocks are (tile_t, tile_h, tile_w) = (2, 8, 8)

    @property
    def nb(self) -> int:
        return _load().lcsa_oracle_blocks_per_frame(self.grid_h, self.grid_w, self.tile_h, self.tile_w)

    @property
    def tokens_per_frame(self) -> int:
        return self.grid_h * self.grid_w


def threads() -> int:
    return _load().lcsa_oracle_threads()


def _tokens_view(x: np.ndarray):
    """x: float32 [tokens][heads][d] (any token/head strides, d contiguous)."""
    assert x.dtype == np.float32 and x.ndim == 3 and x.strides[2] == 4
    return x, x.strides[0] // 4, x.strides[1] // 4


def pool(x: np.ndarray, g: Geometry, n_frames: int) -> np.ndarray:
    """Block means of x -> float64 [heads][(n_frames/tile_t)*nb][d]  (Sec. 3.2)."""
    x, st, sh = _tokens_view(x)
    assert x.shape == (n_frames * g.tokens_per_frame, g.heads, g.head_dim) and n_frames % g.tile_t == 0
    out = np.empty((g.heads, n_frames // g.tile_t * g.nb, g.head_dim), np.float64)
    _load().lcsa_oracle_pool(_p(x, _f32), _cl(st), _cl(sh), _ci(g.heads), _ci(g.head_dim),
                             _ci(n_frames), _ci(g.grid_h), _ci(g.grid_w), _ci(g.tile_t), _ci(g.tile_h), _ci(g.tile_w),
                             _p(out, _f64))
    return out


def scores(pooled_q: np.ndarray, pooled_k: np.ndarray) -> np.ndarray:
    """Coarse block-to-block map S[h][qb][kb] = <q_bar, k_bar>  (Sec. 3.2)."""
    pooled_q = np.ascontiguousarray(pooled_q, np.float64)
    pooled_k = np.ascontiguousarray(pooled_k, np.float64)
    h, n_qb, d = pooled_q.shape
    n_kb = pooled_k.shape[1]
    S = np.empty((h, n_qb, n_kb), np.float64)
    _load().lcsa_oracle_scores(_p(pooled_q, _f64), _p(pooled_k, _f64), _ci(h), _ci(n_qb), _ci(n_kb), _ci(d),
                               _p(S, _f64))
    return S


def allowed(qb: int, kb: int, g: Geometry) -> bool:
    """Spatial local-window predicate on block ids (Sec. 3.3, Fig. 3)."""
    return bool(_load().lcsa_oracle_allowed(_ci(qb), _ci(kb), _ci(g.grid_h), _ci(g.grid_w), _ci(g.tile_h),
                                            _ci(g.tile_w), _ci(g.radius_h), _ci(g.radius_w), _ci(g.window_mode)))


def select(S: np.ndarray, g: Geometry, kv_frames: int):
    """Top-k admissible key blocks per (head, query block): (sel_idx, sel_cnt, gap)."""
    S = np.ascontiguousarray(S, np.float64)
    assert g.q_frames % g.tile_t == 0 and kv_frames % g.tile_t == 0
    n_qb, n_kb = g.q_frames // g.tile_t * g.nb, kv_frames // g.tile_t * g.nb
    assert S.shape == (g.heads, n_qb, n_kb)
    sel_idx = np.empty((g.heads, n_qb, g.topk), np.int32)
    sel_cnt = np.empty((g.heads, n_qb), np.int32)
    gap = np.empty((g.heads, n_qb), np.float64)
    _load().lcsa_oracle_select(_p(S, _f64), _ci(g.heads), _ci(g.q_frames // g.tile_t), _ci(kv_frames // g.tile_t),
                               _ci(g.grid_h), _ci(g.grid_w), _ci(g.tile_h), _ci(g.tile_w),
                               _ci(g.radius_h), _ci(g.radius_w), _ci(g.window_mode), _ci(g.topk),
                               _p(sel_idx, _i32), _p(sel_cnt, _i32), _p(gap, _f64))
    return sel_idx, sel_cnt, gap


def attend(q: np.ndarray, k: np.ndarray, v: np.ndarray, g: Geometry, kv_frames: int,
           sel_idx: np.ndarray, sel_cnt: np.ndarray, scale: float = 0.0, rows=None,
           with_lse: bool = False):
    """Exact softmax attention over the kept blocks (Sec. 3.2, eq. 1).

    q: [q_frames*H*W][heads][d] float32; k, v: [kv_frames*H*W][heads][d] float32
    (oldest visible frame first, the chunk's own frames last).  rows: optional
    int array [[head, qb], ...] restricting the work to those query blocks
    (other entries of the result are NaN).  Returns o float64 [tokens][heads][d]
    (and lse [tokens][heads] if asked).
    """
    q, qst, qsh = _tokens_view(q)
    k, kst, ksh = _tokens_view(k)
    v, vst, vsh = _tokens_view(v)
    assert (kst, ksh) == (vst, vsh) and k.shape == v.shape
    assert q.shape == (g.q_frames * g.tokens_per_frame, g.heads, g.head_dim)
    assert k.shape == (kv_frames * g.tokens_per_frame, g.heads, g.head_dim)
    sel_idx = np.ascontiguousarray(sel_idx, np.int32)
    sel_cnt = np.ascontiguousarray(sel_cnt, np.int32)
    topk = sel_idx.shape[-1]
    assert sel_idx.shape == (g.heads, g.q_frames // g.tile_t * g.nb, topk)
    o = np.full((q.shape[0], g.heads, g.head_dim), np.nan, np.float64)
    lse = np.full((q.shape[0], g.heads), np.nan, np.float64) if with_lse else None
    if rows is None:
        rows_p, n_rows = None, -1
    else:
        rows = np.ascontiguousarray(rows, np.int32).reshape(-1, 2)
        rows_p, n_rows = _p(rows, _i32), rows.shape[0]
    _load().lcsa_oracle_attend(_p(q, _f32), _cl(qst), _cl(qsh), _p(k, _f32), _p(v, _f32), _cl(kst), _cl(ksh),
                               _ci(g.heads), _ci(g.head_dim), _ci(g.q_frames), _ci(kv_frames),
                               _ci(g.grid_h), _ci(g.grid_w), _ci(g.tile_t), _ci(g.tile_h), _ci(g.tile_w),
                               _p(sel_idx, _i32), _p(sel_cnt, _i32), _ci(topk), _f64(scale),
                               rows_p, _ci(n_rows), _p(o, _f64), _p(lse, _f64) if with_lse else None)
    return (o, lse) if with_lse else o


def attend_bwd(q: np.ndarray, k: np.ndarray, v: np.ndarray, d_o: np.ndarray, g: Geometry, kv_frames: int,
               sel_idx: np.ndarray, sel_cnt: np.ndarray, scale: float = 0.0):
    """Gradients of `attend` with the selection held fixed (Sec. 3.2 "Stage 2": the model is trained with the
    sparse attention; the discrete top-k choice carries no gradient): given d_o = dL/do, returns
    (dq [q tokens][heads][d], dk, dv [kv tokens][heads][d]) in float64."""
    q, d_o = np.ascontiguousarray(q, np.float32), np.ascontiguousarray(d_o, np.float32)     # the two share strides
    q, qst, qsh = _tokens_view(q)
    k, kst, ksh = _tokens_view(k)
    v, vst, vsh = _tokens_view(v)
    assert (kst, ksh) == (vst, vsh) and k.shape == v.shape and d_o.shape == q.shape and d_o.dtype == np.float32
    assert q.shape == (g.q_frames * g.tokens_per_frame, g.heads, g.head_dim)
    assert k.shape == (kv_frames * g.tokens_per_frame, g.heads, g.head_dim)
    sel_idx = np.ascontiguousarray(sel_idx, np.int32)
    sel_cnt = np.ascontiguousarray(sel_cnt, np.int32)
    topk = sel_idx.shape[-1]
    dq = np.empty(q.shape, np.float64)
    dk = np.empty(k.shape, np.float64)
    dv = np.empty(k.shape, np.float64)
    _load().lcsa_oracle_attend_bwd(_p(q, _f32), _p(d_o, _f32), _cl(qst), _cl(qsh), _p(k, _f32), _p(v, _f32), _cl(kst), _cl(ksh),
                                   _ci(g.heads), _ci(g.head_dim), _ci(g.q_frames), _ci(kv_frames),
                                   _ci(g.grid_h), _ci(g.grid_w), _ci(g.tile_t), _ci(g.tile_h), _ci(g.tile_w),
                                   _p(sel_idx, _i32), _p(sel_cnt, _i32), _ci(topk), _f64(scale),
                                   _p(dq, _f64), _p(dk, _f64), _p(dv, _f64))
    return dq, dk, dv


def attend_weights(q, k, v, g: Geometry, kv_frames: int, blocks, head: int, q_tok: int, scale: float = 0.0):
    """Softmax weights of one query token over ALL key tokens (zero outside `blocks`) and its output."""
    q, qst, qsh = _tokens_view(q)
    k, kst, ksh = _tokens_view(k)
    v, vst, vsh = _tokens_view(v)
    blocks = np.ascontiguousarray(blocks, np.int32)
    w = np.zeros(kv_frames * g.tokens_per_frame, np.float64)
    o = np.empty(g.head_dim, np.float64)
    _load().lcsa_oracle_attend_weights(_p(q, _f32), _cl(qst), _cl(qsh), _p(k, _f32), _p(v, _f32), _cl(kst), _cl(ksh),
                                       _ci(g.head_dim), _ci(kv_frames), _ci(g.grid_h), _ci(g.grid_w),
                                       _ci(g.tile_t), _ci(g.tile_h), _ci(g.tile_w), _p(blocks, _i32), _ci(len(blocks)),
                                       _f64(scale), _ci(head), _cl(q_tok), _p(o, _f64), _p(w, _f64))
    return w, o


def default_rope_pairs(head_dim: int):
    """Channel pairs given to the (frame, row, column) axes when the caller states no split: a third of the
    pairs to each spatial axis, the rest to the frame axis."""
    third = head_dim // 6
    return head_dim // 2 - 2 * third, third, third


def rope(x: np.ndarray, g: Geometry, n_frames: int, pairs=None, base: float = 10000.0, first_frame: int = 0) -> np.ndarray:
    """Rotary position embedding in its relative formulation (RoFormer, which Sec. 3.3 builds its locality argument
    on), applied per axis of the (frame, row, column) position of a token: the channels of a head are consecutive
    pairs (2i, 2i+1); the first pairs[0] pairs rotate with the frame index (first_frame + frame within x), the next
    pairs[1] with the row, the last pairs[2] with the column; pair i of an axis that owns n pairs turns by the
    angle position * base**(-i/n).  x: [n_frames*H*W][heads][d] -> float64 array of the same shape.  (The paper
    does not print the layout its backbone uses: the split and the base are parameters, their defaults a reading.)"""
    pairs = default_rope_pairs(g.head_dim) if pairs is None else tuple(pairs)
    assert sum(pairs) * 2 == g.head_dim and x.shape == (n_frames * g.tokens_per_frame, g.heads, g.head_dim)
    out = np.empty(x.shape, np.float64)
    x = x.astype(np.float64)
    for tok in range(x.shape[0]):
        f, rem = divmod(tok, g.tokens_per_frame)
        r, c = divmod(rem, g.grid_w)
        pair = 0
        for pos, n in zip((first_frame + f, r, c), pairs):
            for i in range(n):
                angle = pos * base ** (-i / n)
                cs, sn = np.cos(angle), np.sin(angle)
                a, b = x[tok, :, 2 * pair], x[tok, :, 2 * pair + 1]
                out[tok, :, 2 * pair] = a * cs - b * sn
                out[tok, :, 2 * pair + 1] = a * sn + b * cs
                pair += 1
    return out


class SlidingWindowCache:
    """KV cache with sliding-window eviction as a plain list of frames
    (appendix "Discussion on Stream VSR Pipelines"; KV-cache eviction appendix:
    sliding window is the default).  Capacity counts the current chunk's frames."""

    def __init__(self, capacity_frames: int):
        self.capacity = capacity_frames
        self.k_frames: list[np.ndarray] = []
        self.v_frames: list[np.ndarray] = []

    def append(self, k: np.ndarray, v: np.ndarray, n_frames: int) -> None:
        """k, v: [n_frames*H*W][heads][d]; newest frames go to the back, oldest fall off the front."""
        per = k.shape[0] // n_frames
        for f in range(n_frames):
            self.k_frames.append(np.array(k[f * per:(f + 1) * per]))
            self.v_frames.append(np.array(v[f * per:(f + 1) * per]))
        while len(self.k_frames) > self.capacity:
            self.k_frames.pop(0)
            self.v_frames.pop(0)

    @property
    def valid_frames(self) -> int:
        return len(self.k_frames)

    def visible(self):
        """(K, V) of every visible frame, oldest first: [valid_frames*H*W][heads][d]."""
        return np.concatenate(self.k_frames, 0), np.concatenate(self.v_frames, 0)


def block_importance(S: np.ndarray, g: Geometry, kv_frames: int, scale: float = 0.0) -> np.ndarray:
    """Importance of every visible key block, from the coarse block-to-block attention map of one chunk
    (appendix on KV-cache eviction): the map is the softmax (eq. 1, scale 1/sqrt(d)) of the coarse scores
    S (Sec. 3.2) over the key blocks a query block may attend to (Sec. 3.3); the importance of a key
    block is the attention it receives summed over the chunk's query blocks.  [heads][n_kb], fp64."""
    S = np.asarray(S, np.float64)
    n_qb, n_kb = g.q_frames // g.tile_t * g.nb, kv_frames // g.tile_t * g.nb
    assert S.shape == (g.heads, n_qb, n_kb)
    scale = scale if scale > 0 else 1.0 / np.sqrt(g.head_dim)
    imp = np.zeros((g.heads, n_kb))
    for qb in range(n_qb):
        ok = np.array([allowed(qb, kb, g) for kb in range(n_kb)])
        if not ok.any():
            continue
        for h in range(g.heads):
            logit = S[h, qb, ok] * scale
            w = np.exp(logit - logit.max())
            imp[h, ok] += w / w.sum()
    return imp


def group_importance(S: np.ndarray, g: Geometry, kv_frames: int, scale: float = 0.0) -> np.ndarray:
    """Importance of every visible group of tile_t frames = sum over its blocks.  [heads][groups]."""
    imp = block_importance(S, g, kv_frames, scale)
    return imp.reshape(g.heads, kv_frames // g.tile_t, g.nb).sum(axis=-1)


class ImportanceCache:
    """KV cache with importance-based eviction (appendix on KV-cache eviction) as plain lists.

    An entry is one group of tile_t frames.  When new groups do not fit, the cached groups with the
    lowest importance go (equal importance: the older one first); the arriving groups are never
    candidates.  Importance comes from `set_importance` (the coarse map of the chunk attended last)
    and is forgotten at every append: groups that have never been scored count as zero, so without
    scores the cache behaves like a sliding window.  head-wise: every head decides for itself and
    heads may see different frames; uniform: importance is summed over heads and all heads share
    the decision.  Surviving groups stay in temporal order."""

    def __init__(self, capacity_frames: int, tile_t: int, heads: int, uniform: bool):
        assert capacity_frames % tile_t == 0
        self.capacity = capacity_frames // tile_t
        self.tile_t, self.heads, self.uniform = tile_t, heads, uniform
        # per head: list of [k (tokens_per_group, d), v, importance, birth index]
        self.groups: list[list[list]] = [[] for _ in range(heads)]
        self.births = 0

    def set_importance(self, imp: np.ndarray) -> None:
        """imp[heads][visible groups] in temporal order."""
        imp = np.asarray(imp, np.float64)
        assert imp.shape == (self.heads, len(self.groups[0]))
        if self.uniform:
            imp = np.broadcast_to(imp.sum(axis=0, keepdims=True), imp.shape)
        for h in range(self.heads):
            for e, x in zip(self.groups[h], imp[h]):
                e[2] = float(x)

    def victims(self, n_frames: int) -> list[list[int]]:
        """Per head, the visible groups (positions in temporal order, ascending) that an append of n_frames
        frames would drop: lowest importance first, equal importance: the older one first."""
        n_new = n_frames // self.tile_t
        out = []
        for lst in self.groups:
            alive = list(range(len(lst)))
            gone = []
            for _ in range(max(0, len(lst) + n_new - self.capacity)):
                victim = min(alive, key=lambda i: (lst[i][2], i))
                alive.remove(victim)
                gone.append(victim)
            out.append(sorted(gone))
        return out

    def append(self, k: np.ndarray, v: np.ndarray, n_frames: int, victims=None) -> None:
        """victims: per head, the positions to drop instead of the model's own choice (same count).  A test
        passes the decision of the implementation under test here after checking that it is one this
        model's importances allow within the stated near-tie margin, so that both sides keep holding the
        same frames afterwards."""
        assert n_frames % self.tile_t == 0
        n_new = n_frames // self.tile_t
        per = k.shape[0] // n_new
        own = self.victims(n_frames)
        if victims is None:
            victims = own
        for h in range(self.heads):
            lst = self.groups[h]
            assert len(victims[h]) == len(own[h]) and len(set(victims[h])) == len(victims[h])
            for victim in sorted(victims[h], reverse=True):
                lst.pop(victim)
            for e in lst:
                e[2] = 0.0
            for gi in range(n_new):
                lst.append([np.array(k[gi * per:(gi + 1) * per, h]), np.array(v[gi * per:(gi + 1) * per, h]), 0.0,
                            self.births + gi])
        self.births += n_new

    def importances(self) -> np.ndarray:
        """[heads][visible groups]: the importance each visible group currently carries (after set_importance:
        the scores, summed over heads under the uniform policy; after an append: zeros)."""
        return np.array([[e[2] for e in lst] for lst in self.groups], np.float64)

    @property
    def valid_frames(self) -> int:
        return len(self.groups[0]) * self.tile_t

    def birth_order(self) -> np.ndarray:
        """[heads][visible groups]: which appended group (counted from 0) each visible group is."""
        return np.array([[e[3] for e in lst] for lst in self.groups])

    def visible(self):
        """(K, V) as every head sees them, oldest first: [valid_frames*H*W][heads][d]."""
        K = np.stack([np.concatenate([e[0] for e in lst], 0) for lst in self.groups], axis=1)
        V = np.stack([np.concatenate([e[1] for e in lst], 0) for lst in self.groups], axis=1)
        return K, V


def lcsa(q: np.ndarray, k: np.ndarray, v: np.ndarray, g: Geometry, kv_frames: int, rows=None):
    """The whole path on visible K/V: pool -> coarse map -> window + top-k -> attend.

    Returns dict(pooled_q, pooled_k, S, sel_idx, sel_cnt, gap, o)."""
    pq = pool(q, g, g.q_frames)
    pk = pool(k, g, kv_frames)
    S = scores(pq, pk)
    sel_idx, sel_cnt, gap = select(S, g, kv_frames)
    o = attend(q, k, v, g, kv_frames, sel_idx, sel_cnt, rows=rows)
    return dict(pooled_q=pq, pooled_k=pk, S=S, sel_idx=sel_idx, sel_cnt=sel_cnt, gap=gap, o=o)
