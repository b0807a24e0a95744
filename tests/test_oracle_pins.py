"""Pins for the CPU oracle: each test ties one part of oracle/ to something the
paper or plain mathematics fixes, independent of the oracle's own code.

The paper prints no worked numeric example of the attention, so agreement with
the authors' implementation is unpinned; what is pinned is the definition.
"""
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import oracle
from oracle import Geometry

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_qkv(rng, g, kv_frames):
    n = g.grid_h * g.grid_w
    q = rng.standard_normal((g.q_frames * n, g.heads, g.head_dim)).astype(np.float32)
    k = rng.standard_normal((kv_frames * n, g.heads, g.head_dim)).astype(np.float32)
    v = rng.standard_normal((kv_frames * n, g.heads, g.head_dim)).astype(np.float32)
    return q, k, v


def dense_attention(q, k, v, mask=None):
    """Textbook softmax(QK^T/sqrt(d))V per head via library routines; mask[tq][tk] bool."""
    d = q.shape[-1]
    logits = np.einsum("ihc,jhc->hij", q.astype(np.float64), k.astype(np.float64)) / np.sqrt(d)
    if mask is not None:
        logits = np.where(mask[None], logits, -np.inf)
    p = softmax(logits, axis=-1)
    return np.einsum("hij,jhc->ihc", p, v.astype(np.float64)), logsumexp(logits, axis=-1).T


TINY = Geometry(heads=1, head_dim=32, grid_h=6, grid_w=8, tile_h=4, tile_w=4, q_frames=2,
                radius_h=4, radius_w=4, topk=4)


# ---- P1: k = all blocks and unbounded window  ==  dense softmax attention (Sec. 3.2, eq. 1)
@pytest.mark.parametrize("geom,kv_frames", [
    (Geometry(1, 32, 6, 8, 4, 4, 2, -1, -1, 16), 4),        # Tiny grid: half tiles on the bottom row
    (Geometry(3, 8, 5, 7, 2, 3, 1, -1, -1, 3 * 3 * 3), 3),  # ragged in both axes, several heads
    (Geometry(2, 16, 4, 4, 4, 4, 2, -1, -1, 5), 5),         # one tile per frame
])
def test_reduces_to_dense_attention(geom, kv_frames):
    rng = np.random.default_rng(1)
    q, k, v = rand_qkv(rng, geom, kv_frames)
    res = oracle.lcsa(q, k, v, geom, kv_frames)
    assert (res["sel_cnt"] == kv_frames * geom.nb).all()
    want, want_lse = dense_attention(q, k, v)
    np.testing.assert_allclose(res["o"], want, rtol=0, atol=1e-12)
    _, lse = oracle.attend(q, k, v, geom, kv_frames, res["sel_idx"], res["sel_cnt"], with_lse=True)
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=1e-12)


def test_dense_with_strided_head_major_inputs():
    """[heads][tokens][d] storage viewed as [tokens][heads][d] must give the same answer."""
    g = Geometry(2, 8, 4, 6, 2, 3, 1, -1, -1, 8)
    rng = np.random.default_rng(2)
    q, k, v = rand_qkv(rng, g, 2)
    qh, kh, vh = (np.ascontiguousarray(x.transpose(1, 0, 2)).transpose(1, 0, 2) for x in (q, k, v))
    a = oracle.lcsa(q, k, v, g, 2)["o"]
    b = oracle.lcsa(qh, kh, vh, g, 2)["o"]
    np.testing.assert_array_equal(a, b)


# ---- P10: hand-enumerated window sets (Sec. 3.3, Fig. 3)
def load_window_sets():
    out = []
    for line in open(os.path.join(HERE, "golden", "window_sets.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, tiles = line.split(":")
        mode, qt = head.split()
        out.append((mode, int(qt), sorted(int(t) for t in tiles.split())))
    return out


@pytest.mark.parametrize("mode,qt,tiles", load_window_sets())
def test_window_sets_match_hand_enumeration(mode, qt, tiles):
    g = Geometry(1, 4, 12, 16, 4, 4, 2, 4, 4, 1, window_mode={"truncated": 0, "preserved": 1}[mode])
    nb = g.nb
    assert nb == 12
    for qf in range(2):
        for kf in range(3):          # frames play no role
            got = [kt for kt in range(nb) if oracle.allowed(qf * nb + qt, kf * nb + kt, g)]
            assert got == tiles


def test_window_radius_boundaries():
    """Centre distance is a multiple of the tile size: radius 7 -> +-1 tile, 8 -> +-2 (tile 4);
    radius 0 -> same tile position only; odd tile sizes; per-axis radii."""
    def row_reach(radius, tile, n=9, q=4):
        g = Geometry(1, 4, tile * n, 5, tile, 5, 1, radius, -1, 1)
        return [b for b in range(n) if oracle.allowed(q, b, g)]
    assert row_reach(7, 4) == [3, 4, 5]
    assert row_reach(8, 4) == [2, 3, 4, 5, 6]
    assert row_reach(3, 4) == [4]
    assert row_reach(0, 4) == [4]
    assert row_reach(5, 5) == [3, 4, 5]
    assert row_reach(9, 3) == [1, 2, 3, 4, 5, 6, 7]
    # per-axis: rows unbounded, columns radius 0
    g = Geometry(1, 4, 8, 12, 4, 4, 1, -1, 0, 1)
    assert [b for b in range(6) if oracle.allowed(1, b, g)] == [1, 4]
    # the paper-scale window: 8x16 tiles, radius 24 -> +-3 tile rows, +-1 tile column
    g = Geometry(1, 4, 48, 88, 8, 16, 1, 24, 24, 1)
    got = [b for b in range(36) if oracle.allowed(3 * 6 + 2, b, g)]
    assert got == [r * 6 + c for r in range(6) for c in (1, 2, 3)]
    # partial edge tiles use the nominal (unclipped) centre: last column (8 of 16 tokens wide)
    got = [b for b in range(36) if oracle.allowed(0 * 6 + 5, b, g)]
    assert got == [r * 6 + c for r in range(4) for c in (4, 5)]


# ---- P2: k >= n_allowed with a finite window == windowed dense attention
@pytest.mark.parametrize("mode", [0, 1])
def test_windowed_dense_attention(mode):
    g = Geometry(2, 8, 12, 16, 4, 4, 2, 4, 4, 27, window_mode=mode)
    kv_frames = 3
    rng = np.random.default_rng(3)
    q, k, v = rand_qkv(rng, g, kv_frames)
    sets = {(m, qt): t for m, qt, t in load_window_sets()}
    name = "truncated" if mode == 0 else "preserved"
    # token-level mask from the hand-written tile sets (tiles not listed in the fixture are skipped)
    def tile_of(tok):
        r, c = (tok % 192) // 16, tok % 16
        return (r // 4) * 4 + c // 4
    qt = np.array([tile_of(t) for t in range(q.shape[0])])
    kt = np.array([tile_of(t) for t in range(k.shape[0])])
    listed = [t for t in range(12) if (name, t) in sets]
    mask = np.zeros((q.shape[0], k.shape[0]), bool)
    for t in listed:
        mask[np.ix_(qt == t, np.isin(kt, sets[(name, t)]))] = True
    res = oracle.lcsa(q, k, v, g, kv_frames)
    rows = np.isin(qt, listed)
    mask[~rows] = True
    want, _ = dense_attention(q, k, v, mask)
    np.testing.assert_allclose(res["o"][rows], want[rows], rtol=0, atol=1e-12)
    for t in listed:
        for f in range(2):
            assert res["sel_cnt"][0, f * 12 + t] == 3 * len(sets[(name, t)])


# ---- pooling: library mean when tiles divide the grid; closed forms on ragged grids
def test_pool_equals_reshape_mean_when_tiles_divide():
    g = Geometry(3, 5, 8, 12, 4, 3, 2, -1, -1, 1)
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2 * 96, 3, 5)).astype(np.float32)
    want = x.astype(np.float64).reshape(2, 2, 4, 4, 3, 3, 5).mean(axis=(2, 4))   # f,by,bx,h,d
    want = want.transpose(3, 0, 1, 2, 4).reshape(3, 2 * 8, 5)
    np.testing.assert_allclose(oracle.pool(x, g, 2), want, rtol=0, atol=1e-15)


def test_pool_partial_tiles_divide_by_valid_count():
    """x = a*row + b*col + c*frame: the mean over a (possibly clipped) tile is x at its centroid."""
    g = Geometry(1, 1, 6, 8, 4, 3, 2, -1, -1, 1)          # 2 x 3 tiles, bottom row 2 high, right col 2 wide
    f, r, c = np.meshgrid(np.arange(2), np.arange(6), np.arange(8), indexing="ij")
    x = (0.5 * r + 0.25 * c + 2.0 * f).astype(np.float32).reshape(-1, 1, 1)
    got = oracle.pool(x, g, 2).reshape(2, 2, 3)
    rows = [1.5, 4.5]               # centroids of rows {0..3}, {4,5}
    cols = [1.0, 4.0, 6.5]          # centroids of cols {0..2}, {3..5}, {6,7}
    for ff in range(2):
        for by in range(2):
            for bx in range(3):
                assert got[ff, by, bx] == pytest.approx(0.5 * rows[by] + 0.25 * cols[bx] + 2.0 * ff, abs=1e-14)


def test_scores_equal_einsum():
    rng = np.random.default_rng(5)
    pq, pk = rng.standard_normal((2, 7, 9)), rng.standard_normal((2, 11, 9))
    np.testing.assert_allclose(oracle.scores(pq, pk), np.einsum("hqc,hkc->hqk", pq, pk), rtol=0, atol=1e-14)


# ---- top-k: library sort on an unbounded window; P3 invariants under a window
def test_topk_equals_stable_argsort_unbounded():
    g = Geometry(2, 4, 8, 8, 4, 4, 2, -1, -1, 5)
    kv = 3
    rng = np.random.default_rng(6)
    S = rng.standard_normal((2, 2 * 4, kv * 4))
    S[0, 0, :] = np.round(S[0, 0, :])            # force exact ties on one row
    S[1, 3, :] = 0.0                             # and an all-tie row
    idx, cnt, gap = oracle.select(S, g, kv)
    order = np.argsort(-S, axis=-1, kind="stable")   # stable: among equals the lower index first
    want = np.sort(order[..., :5], axis=-1)
    np.testing.assert_array_equal(idx, want)
    assert (cnt == 5).all()
    srt = -np.sort(-S, axis=-1)
    np.testing.assert_allclose(gap, srt[..., 4] - srt[..., 5], rtol=0, atol=0)
    assert gap[1, 3] == 0.0


@pytest.mark.parametrize("mode", [0, 1])
def test_selection_invariants_under_window(mode):
    g = Geometry(2, 4, 20, 28, 4, 4, 2, 6, 9, 7, window_mode=mode)   # 5 x 7 tiles, +-1 rows, +-2 cols
    kv = 4
    nb = g.nb
    rng = np.random.default_rng(7)
    S = rng.standard_normal((2, 2 * nb, kv * nb))
    idx, cnt, gap = oracle.select(S, g, kv)
    for h in range(2):
        for qb in range(2 * nb):
            adm = [kb for kb in range(kv * nb) if oracle.allowed(qb, kb, g)]
            m = min(7, len(adm))
            assert cnt[h, qb] == m
            kept = idx[h, qb, :m]
            assert (idx[h, qb, m:] == -1).all()
            assert (np.diff(kept) > 0).all()                     # ascending, unique
            assert set(kept) <= set(adm)                         # never outside the window
            rest = sorted(set(adm) - set(kept))
            if rest:
                assert S[h, qb, kept].min() >= S[h, qb, rest].max()
                assert gap[h, qb] == pytest.approx(S[h, qb, kept].min() - S[h, qb, rest].max(), abs=0)
            else:
                assert np.isinf(gap[h, qb])


def test_fewer_candidates_than_k_keeps_all_and_pads():
    g = Geometry(1, 4, 8, 8, 4, 4, 1, 0, 0, 6)       # radius 0: only the same tile position
    S = np.random.default_rng(8).standard_normal((1, 4, 3 * 4))
    idx, cnt, gap = oracle.select(S, g, 3)
    for qb in range(4):
        assert cnt[0, qb] == 3
        assert list(idx[0, qb]) == [qb, 4 + qb, 8 + qb, -1, -1, -1]
        assert np.isinf(gap[0, qb])


# ---- P5: Q = 0 -> pure tie-break, and uniform weights over the kept blocks' valid tokens
def test_zero_queries_closed_form():
    g = Geometry(2, 8, 6, 8, 4, 4, 2, 4, 100, 3)      # 2 x 2 tiles/frame; bottom tiles are 2 rows high
    kv = 3
    rng = np.random.default_rng(9)
    q, k, v = rand_qkv(rng, g, kv)
    q[:] = 0.0
    res = oracle.lcsa(q, k, v, g, kv)
    assert (res["sel_idx"] == np.array([0, 1, 2])).all()      # lowest ids: tiles 0,1,2 of the oldest frame
    toks = [r * 8 + c for r in range(4) for c in range(8)] + [r * 8 + c for r in (4, 5) for c in range(4)]
    want = v[toks].astype(np.float64).mean(axis=0)              # [heads][d]
    np.testing.assert_allclose(res["o"], np.broadcast_to(want, res["o"].shape), rtol=0, atol=1e-14)


# ---- P6 / P4: constant V, convexity, weights
def test_constant_v_and_convexity():
    g = TINY
    kv = 4
    rng = np.random.default_rng(10)
    q, k, v = rand_qkv(rng, g, kv)
    res = oracle.lcsa(q, k, v, g, kv)
    vc = np.full_like(v, 0.375)
    o = oracle.attend(q, k, vc, g, kv, res["sel_idx"], res["sel_cnt"])
    np.testing.assert_allclose(o, 0.375, rtol=0, atol=1e-15)
    nb, n = g.nb, g.grid_h * g.grid_w
    for tok in (0, 17, 47, 48 + 40, 95):
        f, r, c = tok // n, (tok % n) // 8, tok % 8
        qb = f * nb + (r // 4) * 2 + c // 4
        blocks = res["sel_idx"][0, qb, :res["sel_cnt"][0, qb]]
        w, o1 = oracle.attend_weights(q, k, v, g, kv, blocks, 0, tok)
        assert w.min() >= 0 and w.sum() == pytest.approx(1.0, abs=1e-14)
        # support = exactly the tokens of the kept blocks
        tiles = np.array([(t // n) * nb + (((t % n) // 8) // 4) * 2 + (t % 8) // 4 for t in range(kv * n)])
        assert ((w > 0) == np.isin(tiles, blocks)).all()
        np.testing.assert_allclose(o1, res["o"][tok, 0], rtol=0, atol=1e-15)
        np.testing.assert_allclose(o1, w @ v[:, 0, :].astype(np.float64), rtol=0, atol=1e-14)
        sup = v[w > 0, 0, :]
        assert (o1 <= sup.max(0) + 1e-15).all() and (o1 >= sup.min(0) - 1e-15).all()


# ---- P7: adding the same vector to every key changes neither selection nor output...
def test_key_shift_invariance_of_attention():
    """...for the exact attention stage (each query's logits all move by the same amount)."""
    g = Geometry(2, 8, 8, 8, 4, 4, 1, 4, 4, 3)
    kv = 2
    rng = np.random.default_rng(11)
    q, k, v = rand_qkv(rng, g, kv)
    # dyadic values so the shifted keys stay exact in float32
    k = np.round(k * 8) / 8
    u = (np.round(rng.standard_normal((1, 2, 8)) * 4) / 4).astype(np.float32)
    res = oracle.lcsa(q, k, v, g, kv)
    o2 = oracle.attend(q, k + u, v, g, kv, res["sel_idx"], res["sel_cnt"])
    np.testing.assert_allclose(o2, res["o"], rtol=0, atol=1e-13)
    # the pooled map moves by a per-row constant, so the selection is unchanged too
    res2 = oracle.lcsa(q, k + u, v, g, kv)
    np.testing.assert_array_equal(res2["sel_idx"], res["sel_idx"])


# ---- P8: a frame duplicated bit for bit ties exactly; the older copy wins
def test_duplicate_frame_tie_prefers_older():
    g = Geometry(1, 8, 8, 8, 4, 4, 1, -1, -1, 2)
    rng = np.random.default_rng(12)
    n = 64
    q = rng.standard_normal((n, 1, 8)).astype(np.float32)
    kf = rng.standard_normal((n, 1, 8)).astype(np.float32)
    k = np.concatenate([kf, kf], 0)
    v = rng.standard_normal((2 * n, 1, 8)).astype(np.float32)
    res = oracle.lcsa(q, k, v, g, 2)
    S = res["S"]
    np.testing.assert_array_equal(S[..., :4], S[..., 4:])
    for qb in range(4):
        best = int(np.argmax(S[0, qb, :4]))
        assert list(res["sel_idx"][0, qb]) == [best, best + 4]   # both copies of the best tile...
    g1 = Geometry(1, 8, 8, 8, 4, 4, 1, -1, -1, 1)
    res1 = oracle.lcsa(q, k, v, g1, 2)
    for qb in range(4):
        assert res1["sel_idx"][0, qb, 0] == int(np.argmax(S[0, qb, :4]))   # ...and with k=1 the older one
        assert res1["gap"][0, qb] == 0.0


# ---- P9: sliding-window cache == the last C frames of the full history
def test_sliding_window_cache_model():
    cap, tq, per = 6, 2, 5
    cache = oracle.SlidingWindowCache(cap)
    hist_k, hist_v = [], []
    rng = np.random.default_rng(13)
    for chunk in range(7):
        k = rng.standard_normal((tq * per, 1, 2)).astype(np.float32)
        v = rng.standard_normal((tq * per, 1, 2)).astype(np.float32)
        cache.append(k, v, tq)
        hist_k.append(k)
        hist_v.append(v)
        allk, allv = np.concatenate(hist_k), np.concatenate(hist_v)
        keep = min((chunk + 1) * tq, cap) * per
        K, V = cache.visible()
        assert cache.valid_frames == keep // per
        np.testing.assert_array_equal(K, allk[-keep:])
        np.testing.assert_array_equal(V, allv[-keep:])
    # odd chunk size against an even capacity: a chunk may straddle the eviction point
    cache = oracle.SlidingWindowCache(4)
    frames = [np.full((per, 1, 2), i, np.float32) for i in range(9)]
    for i in range(0, 9, 3):
        x = np.concatenate(frames[i:i + 3])
        cache.append(x, x, 3)
    assert [int(f[0, 0, 0]) for f in cache.k_frames] == [5, 6, 7, 8]


# ---- scale argument and density sanity
def test_explicit_scale_matches_default_and_changes_result():
    g = Geometry(1, 16, 4, 4, 4, 4, 1, -1, -1, 2)
    rng = np.random.default_rng(14)
    q, k, v = rand_qkv(rng, g, 2)
    res = oracle.lcsa(q, k, v, g, 2)
    a = oracle.attend(q, k, v, g, 2, res["sel_idx"], res["sel_cnt"], scale=0.25)
    np.testing.assert_array_equal(a, res["o"])
    b = oracle.attend(q, k, v, g, 2, res["sel_idx"], res["sel_cnt"], scale=1.0)
    want, _ = dense_attention(q * 4.0, k, v)          # scale 1.0 == logits * sqrt(d)
    np.testing.assert_allclose(b, want, rtol=0, atol=1e-12)


def test_rows_argument_restricts_work():
    g = TINY
    rng = np.random.default_rng(15)
    q, k, v = rand_qkv(rng, g, 4)
    full = oracle.lcsa(q, k, v, g, 4)
    part = oracle.attend(q, k, v, g, 4, full["sel_idx"], full["sel_cnt"], rows=[[0, 3], [0, 6]])
    done = ~np.isnan(part[:, 0, 0])
    # tile 3 of frame 0 = rows 4,5 x cols 4..7 ; tile 2 of frame 1 = rows 4,5 x cols 0..3
    want = sorted([r * 8 + c for r in (4, 5) for c in range(4, 8)] + [48 + r * 8 + c for r in (4, 5) for c in range(4)])
    assert list(np.nonzero(done)[0]) == want
    np.testing.assert_array_equal(part[done], full["o"][done])


# ---- blocks with a temporal extent: the paper's (2, 8, 8) partition (Sec. 3.2) ---------------------
def test_temporal_blocks_reduce_to_dense_attention():
    g = Geometry(2, 8, 5, 6, 2, 4, q_frames=2, radius_h=-1, radius_w=-1, topk=100, tile_t=2)   # ragged in both axes
    kv = 4
    rng = np.random.default_rng(31)
    q, k, v = rand_qkv(rng, g, kv)
    res = oracle.lcsa(q, k, v, g, kv)
    assert res["sel_idx"].shape == (2, 1 * g.nb, 100) and (res["sel_cnt"] == 2 * g.nb).all()
    want, want_lse = dense_attention(q, k, v)
    np.testing.assert_allclose(res["o"], want, rtol=0, atol=1e-12)


def test_temporal_blocks_pool_over_both_frames():
    g = Geometry(1, 3, 4, 6, 2, 3, q_frames=4, radius_h=-1, radius_w=-1, topk=1, tile_t=2)
    x = np.random.default_rng(32).standard_normal((4 * 24, 1, 3)).astype(np.float32)
    want = x.astype(np.float64).reshape(2, 2, 2, 2, 2, 3, 1, 3).mean(axis=(1, 3, 5))   # group, ft, by, r, bx, c, h, d
    want = want.transpose(3, 0, 1, 2, 4).reshape(1, 2 * 4, 3)
    np.testing.assert_allclose(oracle.pool(x, g, 4), want, rtol=0, atol=1e-15)


def test_temporal_blocks_zero_queries_and_window():
    """Q = 0 with (2, 4, 4) blocks on a 6 x 8 grid: kept blocks are the lowest ids of the OLDEST frame pair;
    the window is spatial only, so both frames of a block are always taken together."""
    g = Geometry(1, 8, 6, 8, 4, 4, q_frames=2, radius_h=0, radius_w=4, topk=2, tile_t=2)   # same tile row, +-1 tile column
    kv = 4
    rng = np.random.default_rng(33)
    q, k, v = rand_qkv(rng, g, kv)
    q[:] = 0
    res = oracle.lcsa(q, k, v, g, kv)
    assert g.nb == 4 and res["sel_idx"].shape == (1, 4, 2)
    np.testing.assert_array_equal(res["sel_idx"][0], [[0, 1], [0, 1], [2, 3], [2, 3]])
    # query tile 2 (bottom-left, rows 4,5): kept tiles 2 and 3 of frames 0 and 1 -> rows 4,5 x all 8 columns x 2 frames
    toks = [f * 48 + r * 8 + c for f in (0, 1) for r in (4, 5) for c in range(8)]
    want = v[toks].astype(np.float64).mean(axis=0)[0]
    q_toks = [f * 48 + r * 8 + c for f in (0, 1) for r in (4, 5) for c in range(4)]
    np.testing.assert_allclose(res["o"][q_toks, 0], np.broadcast_to(want, (16, 8)), rtol=0, atol=1e-14)


# ---- importance-based KV eviction (appendix on KV-cache eviction) -------------------------------

def test_importance_unbounded_window_is_softmax_column_mass():
    """With no window the coarse attention map is a plain row softmax of S/sqrt(d) (library routine);
    a key block's importance is its column sum."""
    from scipy.special import softmax
    g = Geometry(3, 16, 8, 12, 4, 4, 2, -1, -1, 4)
    rng = np.random.default_rng(11)
    S = rng.normal(size=(3, 2 * g.nb, 5 * g.nb)) * 7.0
    want = softmax(S / 4.0, axis=-1).sum(axis=1)
    np.testing.assert_allclose(oracle.block_importance(S, g, 5), want, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.block_importance(S, g, 5, scale=0.25), want, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.group_importance(S, g, 5), want.reshape(3, 5, g.nb).sum(-1), rtol=1e-12)
    # a different scale is not the same thing
    assert np.abs(oracle.block_importance(S, g, 5, scale=1.0) - want).max() > 1e-3


def test_importance_zero_scores_closed_form_from_hand_written_windows():
    """S = 0: every query block spreads its unit of attention evenly over the blocks of its window in
    every visible frame; summed per key block with the hand-enumerated 3x4-tile windows."""
    sets = {qt: t for m, qt, t in load_window_sets() if m == "truncated"}
    assert sorted(sets) == list(range(12))
    g = Geometry(2, 4, 12, 16, 4, 4, 2, 4, 4, 1)
    kv = 3
    want = np.zeros(kv * 12)
    for qf in range(2):
        for qt in range(12):
            for f in range(kv):
                for t in sets[qt]:
                    want[f * 12 + t] += 1.0 / (kv * len(sets[qt]))
    got = oracle.block_importance(np.zeros((2, 24, kv * 12)), g, kv)
    np.testing.assert_allclose(got, np.stack([want, want]), rtol=1e-13)


def test_importance_mass_is_conserved_and_stays_in_the_window():
    g = Geometry(2, 8, 12, 16, 4, 4, 2, 0, 0, 1)          # radius 0: a query tile only sees its own tile position
    rng = np.random.default_rng(12)
    kv = 4
    S = rng.normal(size=(2, 24, kv * 12)) * 3.0
    imp = oracle.block_importance(S, g, kv)
    np.testing.assert_allclose(imp.sum(axis=-1), 24.0, rtol=1e-12)      # one unit per query block
    # closed form: softmax over the kv frames of the same tile position
    scale = 1.0 / np.sqrt(8)
    for h in range(2):
        for t in range(12):
            want = np.zeros(kv)
            for qf in range(2):
                z = np.exp(S[h, qf * 12 + t, t::12] * scale)
                want += z / z.sum()
            np.testing.assert_allclose(imp[h, t::12], want, rtol=1e-12)


def _groups(rng, n, per=6, heads=2, d=4):
    return rng.normal(size=(n * per, heads, d)), rng.normal(size=(n * per, heads, d))


@pytest.mark.parametrize("uniform", [False, True])
def test_importance_cache_without_scores_is_the_sliding_window(uniform):
    rng = np.random.default_rng(13)
    a = oracle.ImportanceCache(6, 1, 2, uniform)
    b = oracle.SlidingWindowCache(6)
    for n in (2, 1, 3, 2, 6, 1, 4):
        k, v = _groups(rng, n)
        a.append(k, v, n)
        b.append(k, v, n)
        assert a.valid_frames == b.valid_frames
        for x, y in zip(a.visible(), b.visible()):
            np.testing.assert_array_equal(x, y)


def test_importance_cache_head_wise_and_uniform_decisions():
    rng = np.random.default_rng(14)
    imp = np.array([[3.0, 1.0, 2.0, 5.0], [0.0, 9.0, 9.0, 1.0]])
    want = {False: [[0, 3, 4, 5], [1, 2, 4, 5]],          # every head drops its own two weakest groups
            True: [[1, 2, 4, 5], [1, 2, 4, 5]]}           # sums 3, 10, 11, 6: groups 0 and 3 go for both heads
    for uniform in (False, True):
        c = oracle.ImportanceCache(4, 1, 2, uniform)
        k, v = _groups(rng, 4)
        c.append(k, v, 4)
        c.set_importance(imp)
        k2, v2 = _groups(rng, 2)
        c.append(k2, v2, 2)
        assert c.birth_order().tolist() == want[uniform]
        K, V = c.visible()
        allk = np.concatenate([k, k2])
        for h in range(2):
            np.testing.assert_array_equal(K[:, h], np.concatenate([allk[b * 6:(b + 1) * 6, h] for b in want[uniform][h]]))
        # scores are forgotten at an append: the next eviction without new scores takes the oldest
        k3, v3 = _groups(rng, 1)
        c.append(k3, v3, 1)
        assert c.birth_order().tolist() == [w[1:] + [6] for w in want[uniform]]


def test_importance_cache_ties_evict_the_older_group_and_new_groups_are_safe():
    rng = np.random.default_rng(15)
    c = oracle.ImportanceCache(6, 2, 1, False)            # groups of two frames, room for three groups
    for _ in range(3):
        k, v = _groups(rng, 1, per=12, heads=1)
        c.append(k, v, 2)
    c.set_importance(np.array([[2.0, 2.0, 7.0]]))
    k, v = _groups(rng, 2, per=12, heads=1)
    c.append(k, v, 4)                                     # two groups arrive, two must go: the tied pair, never the arrivals
    assert c.birth_order().tolist() == [[2, 3, 4]]
    assert c.valid_frames == 6


# ---- backward of the attention on the kept pairs (Sec. 3.2 "Stage 2": the model is trained with it) ----------------
# Pinned against a library routine that shares nothing with the oracle: reverse-mode differentiation (torch
# autograd, float64) of the textbook masked softmax attention; against central finite differences of the
# oracle's own forward; and against two identities of eq. (1): the weights of a query sum to one, so the
# gradient it sends to its keys sums to zero over the keys and the gradient it sends to the values sums to dO.

def autograd_attention_grads(q, k, v, d_o, mask=None, scale=None):
    import torch
    tq, tk, tv, tg = (torch.tensor(np.asarray(x, np.float64), requires_grad=r) for x, r in
                      ((q, True), (k, True), (v, True), (d_o, False)))
    scale = 1.0 / np.sqrt(q.shape[-1]) if scale is None else scale
    logits = torch.einsum("ihc,jhc->hij", tq, tk) * scale
    if mask is not None:
        logits = logits.masked_fill(~torch.tensor(mask)[None], float("-inf"))
    o = torch.einsum("hij,jhc->ihc", torch.softmax(logits, dim=-1), tv)
    (o * tg).sum().backward()
    return tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("geom,kv_frames", [
    (Geometry(1, 32, 6, 8, 4, 4, 2, -1, -1, 16), 4),
    (Geometry(3, 8, 5, 7, 2, 3, 1, -1, -1, 27), 3),
])
def test_backward_reduces_to_dense_attention_gradients(geom, kv_frames):
    rng = np.random.default_rng(41)
    q, k, v = rand_qkv(rng, geom, kv_frames)
    d_o = rng.standard_normal(q.shape).astype(np.float32)
    res = oracle.lcsa(q, k, v, geom, kv_frames)
    got = oracle.attend_bwd(q, k, v, d_o, geom, kv_frames, res["sel_idx"], res["sel_cnt"])
    want = autograd_attention_grads(q, k, v, d_o)
    for a, b, name in zip(got, want, ("dq", "dk", "dv")):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-11, err_msg=name)


def token_mask_from_selection(g, kv_frames, sel_idx, sel_cnt, head):
    """mask[q token][k token] of one head, from block ids, written with plain index arithmetic."""
    ty, tx = -(-g.grid_h // g.tile_h), -(-g.grid_w // g.tile_w)
    nb, n = ty * tx, g.grid_h * g.grid_w

    def block_of(tok):
        f, r, c = tok // n, (tok % n) // g.grid_w, tok % g.grid_w
        return (f // g.tile_t) * nb + (r // g.tile_h) * tx + c // g.tile_w
    qb = np.array([block_of(t) for t in range(g.q_frames * n)])
    kb = np.array([block_of(t) for t in range(kv_frames * n)])
    mask = np.zeros((len(qb), len(kb)), bool)
    for b in range(g.q_frames // g.tile_t * nb):
        mask[np.ix_(qb == b, np.isin(kb, sel_idx[head, b, :sel_cnt[head, b]]))] = True
    return mask


@pytest.mark.parametrize("geom,kv_frames", [
    (Geometry(2, 8, 12, 16, 4, 4, 2, 4, 4, 2), 3),                         # window bites, top-k far below the window
    (Geometry(2, 8, 9, 14, 4, 4, 2, 4, 8, 4, window_mode=1, tile_t=2), 4),   # two-frame blocks, clipped tiles, preserved window
])
def test_backward_of_sparse_attention_matches_autograd_with_the_selection_as_a_mask(geom, kv_frames):
    rng = np.random.default_rng(42)
    q, k, v = rand_qkv(rng, geom, kv_frames)
    d_o = rng.standard_normal(q.shape).astype(np.float32)
    res = oracle.lcsa(q, k, v, geom, kv_frames)
    assert (res["sel_cnt"] < kv_frames // geom.tile_t * geom.nb).all()
    dq, dk, dv = oracle.attend_bwd(q, k, v, d_o, geom, kv_frames, res["sel_idx"], res["sel_cnt"])
    for h in range(geom.heads):
        mask = token_mask_from_selection(geom, kv_frames, res["sel_idx"], res["sel_cnt"], h)
        want = autograd_attention_grads(q[:, h:h + 1], k[:, h:h + 1], v[:, h:h + 1], d_o[:, h:h + 1], mask)
        for a, b, name in zip((dq, dk, dv), want, ("dq", "dk", "dv")):
            np.testing.assert_allclose(a[:, h:h + 1], b, rtol=0, atol=1e-11, err_msg=f"{name} head {h}")
    # key tokens of blocks that nobody kept receive exactly nothing
    seen = 0
    for h in range(geom.heads):
        untouched = ~token_mask_from_selection(geom, kv_frames, res["sel_idx"], res["sel_cnt"], h).any(axis=0)
        seen += int(untouched.sum())
        assert (dk[untouched, h] == 0).all() and (dv[untouched, h] == 0).all()
    assert seen > 0 or geom.topk > 2


def test_backward_agrees_with_finite_differences_of_the_forward():
    g = Geometry(1, 4, 6, 6, 4, 4, 1, 4, 4, 2)
    kv_frames = 2
    rng = np.random.default_rng(43)
    q, k, v = rand_qkv(rng, g, kv_frames)
    d_o = rng.standard_normal(q.shape).astype(np.float32)
    sel = oracle.lcsa(q, k, v, g, kv_frames)
    dq, dk, dv = oracle.attend_bwd(q, k, v, d_o, g, kv_frames, sel["sel_idx"], sel["sel_cnt"], scale=0.7)

    def loss(q_, k_, v_):
        return float((oracle.attend(q_, k_, v_, g, kv_frames, sel["sel_idx"], sel["sel_cnt"], scale=0.7) * d_o).sum())
    eps = 2.0 ** -7                           # exactly representable steps keep float32 inputs exact
    for arr, grad, which in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        for _ in range(12):
            idx = tuple(int(rng.integers(s)) for s in arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args_hi, args_lo = [q, k, v], [q, k, v]
            args_hi[which], args_lo[which] = hi, lo
            fd = (loss(*args_hi) - loss(*args_lo)) / (2 * eps)
            assert abs(fd - grad[idx]) < 5e-4 * max(1.0, abs(fd)), (which, idx, fd, grad[idx])


def test_backward_identities_of_the_softmax():
    g = Geometry(2, 8, 10, 12, 4, 4, 2, 4, 4, 3)
    kv_frames = 4
    rng = np.random.default_rng(44)
    q, k, v = rand_qkv(rng, g, kv_frames)
    d_o = rng.standard_normal(q.shape).astype(np.float32)
    sel = oracle.lcsa(q, k, v, g, kv_frames)
    dq, dk, dv = oracle.attend_bwd(q, k, v, d_o, g, kv_frames, sel["sel_idx"], sel["sel_cnt"])
    # sum_j p_ij = 1: the value gradients add up to the upstream gradients, per head and channel
    np.testing.assert_allclose(dv.sum(axis=0), d_o.astype(np.float64).sum(axis=0), rtol=0, atol=1e-10)
    # sum_j u_ij = 0 and dk_j = scale sum_i u_ij q_i: with all queries equal the key gradients cancel over the keys
    q_same = np.broadcast_to(q[:1], q.shape).copy()
    _, dk2, _ = oracle.attend_bwd(q_same, k, v, d_o, g, kv_frames, sel["sel_idx"], sel["sel_cnt"])
    np.testing.assert_allclose(dk2.sum(axis=0), 0.0, atol=1e-10)
    # o does not change when every key moves by the same vector (the logits of a query all shift alike),
    # so dq is orthogonal to nothing in particular but dL along that direction is zero: sum_j dk_j . u = 0 for
    # any u only in the equal-queries case above; for general queries check the directional derivative instead
    u = rng.standard_normal(g.head_dim)
    direction = float((dk * u[None, None, :]).sum())
    contrib = np.einsum("ihc,c->ih", q.astype(np.float64), u)       # every query's logits shift by scale q_i.u: no effect
    assert abs(direction) < 1e-9 * (1 + np.abs(contrib).sum())
    # constant V: o = c whatever the weights, so no gradient reaches q or k
    dq3, dk3, _ = oracle.attend_bwd(q, k, np.full_like(v, 0.5), d_o, g, kv_frames, sel["sel_idx"], sel["sel_cnt"])
    assert np.abs(dq3).max() < 1e-12 and np.abs(dk3).max() < 1e-12


# ---- rotary position embedding per axis (RoFormer's relative formulation, which Sec. 3.3 argues from) ---------------

def test_rope_is_a_complex_phase_per_pair():
    """Library routine as the pin: channel pairs as complex numbers times exp(i * angle)."""
    g = Geometry(2, 12, 3, 5, 2, 2, 2, -1, -1, 1)
    rng = np.random.default_rng(51)
    x = rng.standard_normal((2 * 15, 2, 12)).astype(np.float32)
    pairs, base, first = (2, 1, 3), 100.0, 7
    got = oracle.rope(x, g, 2, pairs, base, first)
    z = x.astype(np.float64).reshape(30, 2, 6, 2) @ np.array([1, 1j])          # [tok][head][pair]
    tok = np.arange(30)
    pos = np.stack([first + tok // 15, (tok % 15) // 5, tok % 5], axis=1).astype(np.float64)     # frame, row, column
    angle = np.concatenate([pos[:, a:a + 1] * base ** (-np.arange(n) / n) for a, n in enumerate(pairs)], axis=1)   # [tok][pair]
    want = z * np.exp(1j * angle)[:, None, :]
    np.testing.assert_allclose(got[..., 0::2], want.real, atol=1e-13)
    np.testing.assert_allclose(got[..., 1::2], want.imag, atol=1e-13)


def test_rope_hand_values_identity_and_norm():
    g = Geometry(1, 6, 2, 3, 1, 1, 1, -1, -1, 1)
    x = np.zeros((6, 1, 6), np.float32)
    x[:, 0, :] = [1, 0, 0, 2, 3, 4]
    out = oracle.rope(x, g, 1, (1, 1, 1), 10000.0, 0)
    np.testing.assert_array_equal(out[0, 0], x[0, 0])                           # frame 0, row 0, column 0: nothing turns
    # token 4 = row 1, column 1: the row pair (0, 2) and the column pair (3, 4) turn by 1 radian, the frame pair stays
    c, s = np.cos(1.0), np.sin(1.0)
    np.testing.assert_allclose(out[4, 0], [1, 0, -2 * s, 2 * c, 3 * c - 4 * s, 3 * s + 4 * c], atol=1e-15)
    np.testing.assert_allclose((out ** 2).sum(-1), (x.astype(np.float64) ** 2).sum(-1), rtol=1e-14)
    # second pair of an axis that owns two pairs turns by position * base**(-1/2)
    g2 = Geometry(1, 4, 1, 9, 1, 1, 1, -1, -1, 1)
    y = np.zeros((9, 1, 4), np.float32)
    y[:, 0, 2] = 1.0
    o2 = oracle.rope(y, g2, 1, (0, 0, 2), 100.0, 0)
    np.testing.assert_allclose(o2[5, 0, 2:], [np.cos(0.5), np.sin(0.5)], atol=1e-15)          # column 5 * 100**-0.5 = 0.5


def test_rope_scores_depend_on_relative_position_only():
    """The property Sec. 3.3 relies on: <rope(q, m), rope(k, n)> is a function of m - n, per axis."""
    g = Geometry(1, 12, 4, 6, 1, 1, 1, -1, -1, 1)
    rng = np.random.default_rng(52)
    qv, kv = rng.standard_normal(12).astype(np.float32), rng.standard_normal(12).astype(np.float32)
    q = np.broadcast_to(qv, (24, 1, 12)).copy()
    k = np.broadcast_to(kv, (24, 1, 12)).copy()
    dots = []
    for first in (0, 5):                                                       # the same content, 5 frames later
        rq, rk = oracle.rope(q, g, 1, None, 10000.0, first), oracle.rope(k, g, 1, None, 10000.0, first)
        dots.append(np.einsum("ihc,jhc->ij", rq, rk))
    np.testing.assert_allclose(dots[0], dots[1], atol=1e-12)
    d = dots[0].reshape(4, 6, 4, 6)                                            # [q row][q col][k row][k col]
    np.testing.assert_allclose(d[0, 0, 1, 2], d[2, 3, 3, 5], atol=1e-12)       # both: one row down, two columns right
    np.testing.assert_allclose(d[1, 4, 0, 1], d[3, 5, 2, 2], atol=1e-12)
    assert abs(d[0, 0, 1, 2] - d[0, 0, 2, 1]) > 1e-3
