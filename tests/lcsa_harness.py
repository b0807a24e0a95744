"""Shared driver for the GPU parity tests: runs one stream of chunks through the HIP
library and through the CPU oracle on identical inputs and compares the results."""
from __future__ import annotations

import sys
from dataclasses import dataclass

import numpy as np
import torch

import oracle
from paper_2510_12747_amd import binding as B
from paper_2510_12747_amd import workloads as wl

NEAR_TIE = 1e-3          # selection may differ from the oracle only where its score gap is below this
OUT_MAX_ABS = 1e-2       # output tolerances from the benchmark definition (unit-variance V)
OUT_MEAN_ABS = 1e-3
IMPORTANCE_RTOL = 2e-4   # group importance: fp32 sums of up to a few thousand softmax weights against fp64
# An eviction decision may differ from the oracle's only among groups whose oracle importances lie within this
# relative band: two values that each carry the relative error asserted above can swap order only if they are
# closer than 2 * IMPORTANCE_RTOL; the band leaves a little room on top of that.
EVICT_NEAR_TIE_REL = 5e-4


def say(msg: str) -> None:
    """Progress line, flushed, so that a run that dies on the GPU still names its case."""
    print(f"[lcsa] {msg}", file=sys.stderr, flush=True)


def to_device(x: np.ndarray, dtype: str, layout: str = "thd") -> torch.Tensor:
    """float32 host array [tokens][heads][d] -> device tensor viewed as [tokens][heads][d].
    layout "thd": token-major storage; "htd": head-major storage (strided view)."""
    if dtype == "bf16":
        t = torch.from_numpy(wl.bf16_bits(x).view(np.int16)).view(torch.bfloat16)
    else:
        t = torch.from_numpy(np.ascontiguousarray(x, np.float32))
    if layout == "htd":
        return t.permute(1, 0, 2).contiguous().cuda().permute(1, 0, 2)
    return t.cuda()


def geoms(w: wl.Workload, topk=None, radius=None, window_mode=0, tile_t=1):
    """(library geometry, oracle geometry) of a workload."""
    k = w.topk if topk is None else topk
    r = w.radius if radius is None else radius
    rh, rw = (r, r) if np.isscalar(r) else r
    g = B.Geom(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames, w.cache_frames,
               rh, rw, k, dtype=B.LCSA_BF16 if w.dtype == "bf16" else B.LCSA_F32, window_mode=window_mode,
               tile_t=tile_t)
    og = oracle.Geometry(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, w.q_frames, rh, rw, k,
                         window_mode=window_mode, tile_t=tile_t)
    return g, og


def sample_rows(og: oracle.Geometry, n_random: int, seed: int = 0) -> np.ndarray:
    """(head, query block) rows to verify at sizes where the oracle cannot do them all:
    every corner / edge-centre tile of each query frame for head 0 and the last head, plus random rows."""
    ty = -(-og.grid_h // og.tile_h)
    tx = -(-og.grid_w // og.tile_w)
    nb = ty * tx
    tiles = {(by, bx) for by in (0, ty // 2, ty - 1) for bx in (0, tx // 2, tx - 1)}
    q_groups = og.q_frames // og.tile_t
    rows = {(h, f * nb + by * tx + bx) for h in {0, og.heads - 1} for f in range(q_groups) for by, bx in tiles}
    rng = np.random.default_rng(seed)
    while len(rows) < len(tiles) * q_groups * len({0, og.heads - 1}) + n_random:
        rows.add((int(rng.integers(og.heads)), int(rng.integers(q_groups * nb))))
    return np.array(sorted(rows), np.int32)


@dataclass
class StepResult:
    sel_mismatch_rows: int       # rows whose set differs from the oracle's (all of them near-ties, else assert)
    near_tie_rows: int           # rows with oracle gap < NEAR_TIE
    max_abs: float
    mean_abs: float
    rows_checked: int


def check_selection(sel_idx, sel_cnt, o_idx, o_cnt, o_gap, og, kv_frames, S):
    """Bit-exact selection except rows whose oracle gap is below NEAR_TIE; every GPU row must
    still be a valid selection (ascending, unique, admissible, right count, -1 padded), and on a
    row that differs the exchange must be one the oracle's own fp64 scores S allow: every block
    the GPU kept scores at least S_(k) - NEAR_TIE and every block of the oracle's set that the
    GPU left out scores at most S_(k) + NEAR_TIE, S_(k) being the oracle's weakest kept score."""
    sel_idx, sel_cnt = sel_idx.cpu().numpy(), sel_cnt.cpu().numpy()
    np.testing.assert_array_equal(sel_cnt, o_cnt)
    diff = (sel_idx != o_idx).any(axis=-1)
    near = o_gap < NEAR_TIE
    bad = diff & ~near
    assert not bad.any(), f"{bad.sum()} rows differ from the oracle with gap >= {NEAR_TIE}: first {np.argwhere(bad)[:5]}"
    for h, qb in np.argwhere(diff):
        assert_valid_near_tie_row(sel_idx[h, qb], int(sel_cnt[h, qb]), o_idx[h, qb], S[h, qb], int(qb), og, kv_frames)
    return sel_idx, sel_cnt, int(diff.sum()), int(near.sum())


def assert_valid_near_tie_row(got_ids, m, oracle_ids, s_row, qb, og, kv_frames):
    """A row whose kept set differs from the oracle's: structure, admissibility, and the score bounds
    that make it an exchange among near-tied blocks (s_row = the oracle's fp64 scores of the row)."""
    kept = got_ids[:m]
    assert (np.diff(kept) > 0).all() and (got_ids[m:] == -1).all()
    assert kept.min() >= 0 and kept.max() < kv_frames // og.tile_t * og.nb
    assert all(oracle.allowed(qb, int(kb), og) for kb in kept)
    want = oracle_ids[:m]
    s_k = s_row[want].min()                                # the oracle's weakest kept score
    extra = np.setdiff1d(kept, want)                       # kept by the GPU only
    lost = np.setdiff1d(want, kept)                        # kept by the oracle only
    assert len(extra) == len(lost) > 0
    assert (s_row[extra] >= s_k - NEAR_TIE).all(), f"row {qb}: kept block scores {s_row[extra]} below S_k {s_k} - {NEAR_TIE}"
    assert (s_row[lost] <= s_k + NEAR_TIE).all(), f"row {qb}: dropped block scores {s_row[lost]} above S_k {s_k} + {NEAR_TIE}"


def check_outputs(o_gpu: torch.Tensor, q, K, V, og, kv_frames, sel_idx, sel_cnt, rows, scale=0.0,
                  max_abs=OUT_MAX_ABS, mean_abs=OUT_MEAN_ABS, bf16_relative=False, large_v=False):
    """Compares against the oracle's attention on the SAME selection (the GPU's, which equals the
    oracle's except on reported near-tie rows).

    bf16_relative: for shapes where a row attends to a handful of keys (tiny clipped blocks, sharp softmax rows)
    |o| reaches 4 and more and the rounding of O to bf16 alone (half an ulp = up to 2^-8 |o|) exceeds max_abs;
    the bound is then 2^-8 |o| + 2e-3 per element (rounding of the result + everything inside the kernel), and
    the mean bound grows by the mean rounding error of the result, a quarter ulp <= 2^-9 |o|.

    large_v (with bf16_relative): V far from unit variance.  What happens inside the kernel then scales with the
    values averaged, not with the result: probabilities enter the second product rounded to half (relative 2^-11
    each), so the per-element bound gains 2^-10 * sum_j p_j |v_j|, the attention of |V| taken from the oracle."""
    want = oracle.attend(q, K, V, og, kv_frames, sel_idx, sel_cnt, scale=scale, rows=rows)
    got = o_gpu.float().cpu().numpy().astype(np.float64)
    done = ~np.isnan(want)
    assert done.any()
    err = np.abs(got - want)[done]
    assert np.isfinite(got[done]).all()
    if bf16_relative:
        bound = 2.0 ** -8 * np.abs(want[done]) + 2e-3
        if large_v:
            bound += 2.0 ** -10 * oracle.attend(q, K, np.abs(V), og, kv_frames, sel_idx, sel_cnt, scale=scale, rows=rows)[done]
        worst = int(np.argmax(err - bound))
        assert (err <= bound).all(), f"error {err[worst]:.3e} at |o| = {abs(want[done][worst]):.3f} exceeds {bound[worst]:.3e}"
        mean_bound = mean_abs + 2.0 ** -9 * np.abs(want[done]).mean() + (bound.mean() if large_v else 0.0)
        assert err.mean() <= mean_bound, f"mean-abs {err.mean():.3e} > {mean_bound:.3e}"
        return float(err.max()), float(err.mean())
    worst = int(np.argmax(err))
    assert err.max() <= max_abs, f"max-abs {err.max():.3e} > {max_abs} (at |o| = {abs(want[done][worst]):.3f})"
    assert err.mean() <= mean_abs, f"mean-abs {err.mean():.3e} > {mean_abs}"
    return float(err.max()), float(err.mean())


def check_eviction(got, own, imp, uniform, rel=EVICT_NEAR_TIE_REL) -> int:
    """got / own: per head, the positions (temporal order) dropped by the implementation under test / by the
    oracle's model; imp[heads][groups]: the oracle's importances the decision was taken on.  The two may differ
    only by an exchange among groups whose oracle importances lie within the relative band `rel` (equal
    importances, e.g. a cache that was never scored, admit no exchange: the older group goes).  Returns the
    number of heads decided differently."""
    if uniform:
        assert all(g == got[0] for g in got), f"uniform policy: heads decided differently: {got}"
    differing = 0
    for h, (a, b) in enumerate(zip(got, own)):
        assert len(a) == len(b) and len(set(a)) == len(a), f"head {h}: dropped {a}, the oracle drops {b}"
        if sorted(a) == sorted(b):
            continue
        differing += 1
        swapped = sorted(set(a) ^ set(b))
        lo, hi = imp[h, swapped].min(), imp[h, swapped].max()
        assert hi > lo, f"head {h}: dropped {a} instead of {b} although the groups tie exactly (older goes first)"
        assert hi - lo <= rel * hi, (f"head {h}: dropped {a}, the oracle drops {b}; importances of the exchanged "
                                     f"groups {imp[h, swapped]} are further apart than {rel} relative")
    return differing


class Pipeline:
    """One layer's state on both sides: the library's cache and the oracle's list model."""

    def __init__(self, w: wl.Workload, layer: int = 0, layout: str = "thd", eviction: int = B.LCSA_EVICT_SLIDING, **geom_kw):
        self.w, self.layout = w, layout
        self.g, self.og = geoms(w, **geom_kw)
        self.stream = wl.ChunkStream(w, layer)
        self.cache = B.lcsa_cache_init(self.g)
        self.eviction = eviction
        if eviction == B.LCSA_EVICT_SLIDING:
            self.model = oracle.SlidingWindowCache(w.cache_frames)
        else:
            B.lcsa_cache_set_eviction(self.cache, eviction)
            self.model = oracle.ImportanceCache(w.cache_frames, self.g.tile_t, w.heads,
                                                eviction == B.LCSA_EVICT_IMPORTANCE_UNIFORM)
        self.chunk = 0

    def feed(self, q=None, k=None, v=None):
        """Appends the next chunk on both sides; returns (q host, q device)."""
        if q is None:
            q, k, v = self.stream.next()
        w = self.w
        kd, vd = to_device(k, w.dtype, self.layout), to_device(v, w.dtype, self.layout)
        if isinstance(self.model, oracle.ImportanceCache):
            # The library decides on the device which groups leave.  Its decision is read back from the slot
            # table, checked against what the oracle's fp64 importances allow, and the model then drops the
            # same groups, so that a near-tie decided the other way does not end the comparison.
            n = self.model.valid_frames // self.g.tile_t
            before = B.lcsa_cache_order(self.cache).cpu().numpy().copy()
            B.lcsa_kv_cache_append(self.cache, kd, vd, w.q_frames)
            after = B.lcsa_cache_order(self.cache).cpu().numpy()
            own = self.model.victims(w.q_frames)
            m = n - len(own[0])
            got = [[i for i in range(n) if before[h, i] not in set(after[h, :m].tolist())] for h in range(self.g.heads)]
            self.near_tie_evictions = getattr(self, "near_tie_evictions", 0) + check_eviction(
                got, own, self.model.importances(), self.eviction == B.LCSA_EVICT_IMPORTANCE_UNIFORM)
            self.model.append(k, v, w.q_frames, victims=got)
        else:
            self.model.append(k, v, w.q_frames)
            B.lcsa_kv_cache_append(self.cache, kd, vd, w.q_frames)
        assert B.lcsa_cache_valid_frames(self.cache) == self.model.valid_frames
        self.chunk += 1
        return q, to_device(q, w.dtype, self.layout)

    def check_pooled_k(self, tol=2e-5):
        K, _ = self.model.visible()
        want = oracle.pool(K, self.og, self.model.valid_frames)
        got = B.lcsa_cache_pooled_k(self.cache).cpu().numpy()
        nb, tt = self.g.nb, self.g.tile_t
        order = B.lcsa_cache_order(self.cache)
        order = None if order is None else order.cpu().numpy()
        for grp in range(self.model.valid_frames // tt):
            if order is None:
                s = B.lcsa_cache_frame_slot(self.cache, grp * tt)
                np.testing.assert_allclose(got[:, s * nb:(s + 1) * nb], want[:, grp * nb:(grp + 1) * nb], rtol=0, atol=tol)
            else:       # every head has its own table of slots (and may hold different frames)
                for h in range(self.g.heads):
                    s = int(order[h, grp])
                    np.testing.assert_allclose(got[h, s * nb:(s + 1) * nb], want[h, grp * nb:(grp + 1) * nb], rtol=0, atol=tol)
        if order is not None:   # a head's visible groups sit in distinct slots
            n = self.model.valid_frames // tt
            assert all(len(set(order[h, :n])) == n and order[h, :n].max() < self.g.cache_frames // tt for h in range(self.g.heads))

    def score_groups(self, q, qd, rtol=IMPORTANCE_RTOL):
        """lcsa_block_importance against the oracle's importance of the visible groups; the oracle's own
        values drive the model's next eviction.  Returns the oracle's importance."""
        pq = B.lcsa_pool_blocks(self.g, qd, self.g.q_frames)
        got = B.lcsa_block_importance(self.g, pq, self.cache).cpu().numpy()
        kvf = self.model.valid_frames
        K, _ = self.model.visible()
        S = oracle.scores(oracle.pool(q, self.og, self.g.q_frames), oracle.pool(K, self.og, kvf))
        want = oracle.group_importance(S, self.og, kvf)
        n = kvf // self.g.tile_t
        np.testing.assert_allclose(got[:, :n], want, rtol=rtol, atol=1e-5)
        assert (got[:, n:] == 0).all()
        np.testing.assert_allclose(got.sum(axis=1), self.g.n_qb, rtol=1e-4)     # one unit of attention per query block
        if isinstance(self.model, oracle.ImportanceCache):
            self.model.set_importance(want)
        return want

    def step(self, q, qd, rows=None, g=None, og=None, scale=0.0, max_abs=OUT_MAX_ABS, mean_abs=OUT_MEAN_ABS,
             check_lse=False, bf16_relative=False) -> StepResult:
        """pool -> select -> attend on the GPU, the same on the oracle, compare."""
        g = g or self.g
        og = og or self.og
        kvf = self.model.valid_frames
        K, V = self.model.visible()
        pq = B.lcsa_pool_blocks(g, qd, g.q_frames)
        sel_idx, sel_cnt, gap = B.lcsa_select_blocks(g, pq, self.cache)
        # the fused call must give the very same bits as the two calls
        f_pq, f_idx, f_cnt, f_gap = B.lcsa_pool_select_blocks(g, qd, self.cache)
        assert torch.equal(f_pq, pq) and torch.equal(f_idx, sel_idx) and torch.equal(f_cnt, sel_cnt) and torch.equal(f_gap, gap)
        lse = torch.empty(qd.shape[0], g.heads, dtype=torch.float32, device="cuda") if check_lse else None
        o = B.lcsa_sparse_attn_fwd(g, qd, self.cache, sel_idx, sel_cnt, lse=lse, scale=scale)
        torch.cuda.synchronize()
        o_pq = oracle.pool(q, og, g.q_frames)
        np.testing.assert_allclose(pq.cpu().numpy(), o_pq, rtol=0, atol=2e-5)
        S = oracle.scores(o_pq, oracle.pool(K, og, kvf))
        o_idx, o_cnt, o_gap = oracle.select(S, og, kvf)
        s_idx, s_cnt, n_diff, n_near = check_selection(sel_idx, sel_cnt, o_idx, o_cnt, o_gap, og, kvf, S)
        ggap = gap.cpu().numpy()
        fin = np.isfinite(o_gap)
        assert (np.isinf(ggap) == ~fin).all()
        np.testing.assert_allclose(ggap[fin], o_gap[fin], rtol=0, atol=1e-3)
        mx, mean = check_outputs(o, q, K, V, og, kvf, s_idx, s_cnt, rows, scale, max_abs, mean_abs, bf16_relative)
        if check_lse:
            _, want_lse = oracle.attend(q, K, V, og, kvf, s_idx, s_cnt, scale=scale, rows=rows, with_lse=True)
            done = ~np.isnan(want_lse)
            np.testing.assert_allclose(lse.cpu().numpy()[done], want_lse[done], rtol=0, atol=2e-3)
        n_rows = g.heads * g.n_qb if rows is None else len(rows)
        return StepResult(n_diff, n_near, mx, mean, n_rows)
