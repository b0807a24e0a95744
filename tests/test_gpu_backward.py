"""GPU parity of lcsa_sparse_attn_bwd against the oracle's fp64 gradients (selection held fixed), through the
same pipeline a training step would run: append, pool + select, forward (output and LSE), backward.

Tolerances.  The kernels compute in float from the stored element type with fixed summation orders; what
separates them from the oracle is (1) float accumulation over up to a few thousand terms (relative ~1e-6 each),
and (2) the forward's LSE (float sums of float exponentials on both forward paths: absolute ~2e-6).  The
forward's OUTPUT does not enter: D_i = dO_i.o_i is formed from the kernel's own probabilities (with o rounded to
bf16 it would be off by up to 4e-2 here and d_q, d_k by 6e-3 of their largest value).  Bars, for f32 and bf16 data
alike: max-abs <= 2e-5 and mean-abs <= 2e-6, both relative to the largest magnitude of the gradient compared
(gradients have no fixed scale of their own).

The matrix-core kernels (bf16, d = 128, 128-token blocks) round p_ij and u_ij to bf16 (relative 2^-9 each) before
the second-level products: an element of a gradient is a sum of such terms, its error at most 2^-9 sum |term| and
typically that over the square root of the number of terms.  Bars: max-abs <= 6e-3 and mean-abs <= 6e-4 of the
largest magnitude; D_i itself is formed in float from unrounded p and t and keeps the float bar."""
import numpy as np
import pytest
import torch

import oracle
from lcsa_harness import Pipeline, check_selection, say, to_device
from paper_2510_12747_amd import binding as B
from paper_2510_12747_amd import workloads as wl

pytestmark = pytest.mark.gpu

BARS = {"float": (2e-5, 2e-6),        # float FMA kernels, f32 and bf16 data alike
        "matrix": (6e-3, 6e-4)}       # matrix-core kernels: p and u enter the second-level products rounded to bf16


def run_backward(w, chunks=None, seed=0, d_o_layout="thd", **kw):
    p = Pipeline(w, **kw)
    for _ in range(w.prime_chunks + 1 if chunks is None else chunks):
        q, qd = p.feed()
    g, og = p.g, p.og
    kvf = p.model.valid_frames
    K, V = p.model.visible()
    pq, sel_idx, sel_cnt, gap = B.lcsa_pool_select_blocks(g, qd, p.cache)
    lse = torch.empty(qd.shape[0], g.heads, dtype=torch.float32, device="cuda")
    B.lcsa_sparse_attn_fwd(g, qd, p.cache, sel_idx, sel_cnt, lse=lse)
    rng = np.random.default_rng(100 + seed)
    d_o = rng.standard_normal(q.shape).astype(np.float32)
    if w.dtype == "bf16":
        d_o = wl.round_to_bf16(d_o)
    Kd, Vd, gd = to_device(K, w.dtype), to_device(V, w.dtype), to_device(d_o, w.dtype, d_o_layout)
    # the selection the gradients are taken on is the library's; it must be the oracle's up to reported near-ties
    S = oracle.scores(oracle.pool(q, og, g.q_frames), oracle.pool(K, og, kvf))
    o_idx, o_cnt, o_gap = oracle.select(S, og, kvf)
    s_idx, s_cnt, n_diff, _ = check_selection(sel_idx, sel_cnt, o_idx, o_cnt, o_gap, og, kvf, S)
    want = oracle.attend_bwd(q, K, V, d_o, og, kvf, s_idx, s_cnt)
    o_ref = oracle.attend(q, K, V, og, kvf, s_idx, s_cnt)
    D_ref = (d_o.astype(np.float64) * o_ref).sum(axis=-1)            # D_i by its definition g_i . o_i on the exact output
    matrix_cores = w.dtype == "bf16" and w.head_dim == 128 and g.tile_t * g.tile_h * g.tile_w == 128
    results = None
    for float_path in ([False, True] if matrix_cores else [True]):
        dq, dk, dv, delta = B.lcsa_sparse_attn_bwd(g, qd, Kd, Vd, kvf, sel_idx, sel_cnt, gd, lse, float_path=float_path)
        torch.cuda.synchronize()
        np.testing.assert_allclose(delta.cpu().numpy(), D_ref, rtol=0, atol=BARS["float"][0] * max(1.0, np.abs(D_ref).max()))
        max_bar, mean_bar = BARS["float" if float_path else "matrix"]
        out = {}
        for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), want):
            got = got.cpu().numpy().astype(np.float64)
            assert np.isfinite(got).all()
            size = np.abs(ref).max()
            err = np.abs(got - ref)
            assert err.max() <= max_bar * size, f"{name}: max-abs {err.max():.3e} > {max_bar} x {size:.3f} (float_path={float_path})"
            assert err.mean() <= mean_bar * size, f"{name}: mean-abs {err.mean():.3e} > {mean_bar} x {size:.3f} (float_path={float_path})"
            # tokens of key blocks that nobody kept get exactly zero
            assert ((ref == 0) <= (got == 0)).all(), f"{name}: nonzero where the oracle's gradient is exactly zero"
            out[name] = (err.max() / size, err.mean() / size)
        say(f"{w.name} backward ({'float' if float_path else 'matrix cores'}): selection differs on {n_diff} rows; relative max / mean error " +
            ", ".join(f"{n} {a:.1e} / {b:.1e}" for n, (a, b) in out.items()))
        if results is None:
            results = (dq, dk, dv)
    return results


def test_backward_tiny_f32():
    run_backward(wl.WORKLOADS["tiny"])


def test_backward_f32_window_bites_and_temporal_blocks():
    w = wl.with_overrides(wl.WORKLOADS["tiny"], name="bwd-f32", heads=2, grid_h=14, grid_w=18, radius=4, topk=5)
    run_backward(w)
    run_backward(wl.with_overrides(w, grid_h=10, grid_w=14, topk=3), tile_t=2, window_mode=1)


def test_backward_small_video_bf16():
    """bf16 inputs, d = 128, 128-token blocks: the forward runs on the matrix-core kernel (LSE from half-precision
    probabilities), the backward reads the raster tensors."""
    run_backward(wl.with_overrides(wl.WORKLOADS["small"], name="bwd-small", heads=3))


def test_backward_paper_scale_grid():
    """The paper-scale grid (48 x 88 tokens, 36 blocks per frame of which the last column is clipped to 8 of 16
    columns, 2 query + 4 cached frames, top-k 32 inside the 24-token window) with 4 of the 12 heads: 288 query-side
    and 864 key-side workgroups, several rounds on 256 compute units, in the launch arithmetic the benchmark times.
    (All 12 heads would keep the oracle busy for minutes; heads are independent of each other.)"""
    say("backward at the paper-scale grid: the oracle's fp64 gradients take about half a minute")
    run_backward(wl.with_overrides(wl.WORKLOADS["paper"], name="bwd-paper-grid", heads=4))


def test_backward_clipped_blocks_and_partly_filled_cache():
    w = wl.with_overrides(wl.WORKLOADS["small"], name="bwd-edge", heads=2, grid_h=20, grid_w=40, radius=16, topk=6)
    run_backward(w, chunks=2)                                   # 4 of 6 frames visible
    run_backward(wl.with_overrides(w, tile_h=8, tile_w=8, grid_h=21, grid_w=37, topk=9), tile_t=2, seed=1)


def test_backward_each_tensor_with_strides_of_its_own():
    """q token-major, dO head-major, K and V token-major: every tensor of the call is addressed through its own strides
    (on the matrix cores the key-side kernel has a build of its own for Q and dO that do not share theirs)."""
    w = wl.with_overrides(wl.WORKLOADS["small"], name="bwd-strides", heads=2, grid_h=20, grid_w=40, radius=16, topk=6)
    run_backward(w, d_o_layout="htd")


def test_backward_generic_bf16_d64():
    w = wl.with_overrides(wl.WORKLOADS["small"], name="bwd-d64", heads=2, head_dim=64, grid_h=10, grid_w=20,
                          tile_h=4, tile_w=8, radius=8, topk=5)
    run_backward(w)


def test_backward_is_deterministic_and_rejects_bad_arguments():
    w = wl.with_overrides(wl.WORKLOADS["small"], name="bwd-det", heads=2, grid_h=16, grid_w=32, topk=4)
    a = run_backward(w)
    b = run_backward(w)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    g = B.Geom(2, 128, 16, 32, 8, 16, 2, 6, 16, 16, 4)
    t = torch.zeros(2 * 16 * 32, 2, 128, dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros(6 * 16 * 32, 2, 128, dtype=torch.bfloat16, device="cuda")
    si = torch.zeros(2, g.n_qb, 4, dtype=torch.int32, device="cuda")
    sc = torch.zeros(2, g.n_qb, dtype=torch.int32, device="cuda")
    lse = torch.zeros(t.shape[0], 2, device="cuda")
    with pytest.raises(B.LcsaError):
        B.lcsa_sparse_attn_bwd(g, t, kv, kv, 1, si, sc, t, lse)      # fewer key frames than the chunk has
    dq, dk, dv, _ = B.lcsa_sparse_attn_bwd(g, t, kv, kv, 6, si, sc, t, lse)   # nothing kept anywhere: all zeros
    assert not dq.any() and not dk.any() and not dv.any()
