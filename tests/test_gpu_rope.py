"""GPU parity of lcsa_rope_pool_blocks (rotary embedding per axis fused with the block pooling) against the oracle.

The rotated tokens are float results rounded to the element type: against the oracle's fp64 rotation they may
differ by the rounding itself (half an ulp: 2^-9 relative for bf16) plus, where the float and the fp64 value fall
on different sides of a rounding boundary, one more ulp: 2^-7 |x| for bf16 (one ulp and a half), nothing for
f32; on top of that the float rotation itself: a component a cos - b sin carries an error relative to the size of
its PAIR (a, b), not to its own size (it may cancel to nothing): 4e-6 of the pair's norm, which covers float
sines and cosines of angles up to thousands of radians (frequency accurate to ~2e-7 relative).  The
pooled means are held to the pooling bar (2e-5) against the oracle's pooling of the tokens the kernel STORED,
and must be the very bits lcsa_pool_blocks gives on them."""
import numpy as np
import pytest
import torch

import oracle
from lcsa_harness import say, to_device
from paper_2510_12747_amd import binding as B
from paper_2510_12747_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_rope(w, n_frames, pairs, base, first_frame, tile_t=1, layout="thd"):
    g = B.Geom(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, n_frames, n_frames, w.radius, w.radius, w.topk,
               dtype=B.LCSA_BF16 if w.dtype == "bf16" else B.LCSA_F32, tile_t=tile_t)
    og = oracle.Geometry(w.heads, w.head_dim, w.grid_h, w.grid_w, w.tile_h, w.tile_w, n_frames, w.radius, w.radius, w.topk, tile_t=tile_t)
    rng = np.random.default_rng(7)
    x = rng.standard_normal((n_frames * w.tokens_per_frame, w.heads, w.head_dim)).astype(np.float32) * 2
    if w.dtype == "bf16":
        x = wl.round_to_bf16(x)
    xd = to_device(x, w.dtype, layout)
    x_rot, pooled = B.lcsa_rope_pool_blocks(g, xd, n_frames, pairs, base, first_frame)
    torch.cuda.synchronize()
    want = oracle.rope(x, og, n_frames, pairs, base if base > 0 else 10000.0, first_frame)
    got = x_rot.float().cpu().numpy()
    norm = np.repeat(np.sqrt((x.astype(np.float64).reshape(x.shape[0], x.shape[1], -1, 2) ** 2).sum(-1)), 2, axis=-1)   # of each channel's pair
    bound = (2.0 ** -7 * np.abs(want) if w.dtype == "bf16" else 0.0) + 4e-6 * norm + 1e-7
    err = np.abs(got - want)
    assert (err <= bound).all(), f"rotated tokens: error {err.max():.3e}"
    # pooling: of the stored tokens, to the pooling bar; and the bits of lcsa_pool_blocks on them
    np.testing.assert_allclose(pooled.cpu().numpy(), oracle.pool(got, og, n_frames), rtol=0, atol=2e-5)
    assert torch.equal(pooled, B.lcsa_pool_blocks(g, x_rot, n_frames))
    # in place
    x_in = xd.clone()
    same, pooled2 = B.lcsa_rope_pool_blocks(g, x_in, n_frames, pairs, base, first_frame, x_rot=x_in)
    assert same is x_in and torch.equal(x_in, x_rot) and torch.equal(pooled2, pooled)
    say(f"rope {w.name}: max error {err.max():.2e} at |x| up to {np.abs(want).max():.1f}")


def test_rope_pool_bf16_small_grid_default_split():
    w = wl.with_overrides(wl.WORKLOADS["small"], name="rope-small", heads=3)
    run_rope(w, 2, oracle.default_rope_pairs(128), 0.0, 5)


def test_rope_pool_bf16_clipped_two_frame_blocks_head_major():
    w = wl.with_overrides(wl.WORKLOADS["small"], name="rope-2x8x8", heads=2, grid_h=21, grid_w=37, tile_h=8, tile_w=8)
    run_rope(w, 4, (10, 30, 24), 500.0, 0, tile_t=2, layout="htd")


def test_rope_pool_large_positions():
    """Columns up to 239 and frame indices beyond 4000: angles of thousands of radians on the first pairs."""
    w = wl.with_overrides(wl.WORKLOADS["small"], name="rope-wide", heads=1, grid_h=8, grid_w=240)
    run_rope(w, 1, oracle.default_rope_pairs(128), 10000.0, 4321)


def test_rope_pool_f32_tiny():
    w = wl.WORKLOADS["tiny"]
    run_rope(w, 2, (6, 5, 5), 10000.0, 3)
    run_rope(w, 2, (16, 0, 0), 100.0, 0)             # one axis owns everything


def test_rope_pool_wide_tiles_without_the_table():
    """The kernel keeps the (cosine, sine) values of a block in an LDS table of at most 4096 entries; a block
    with more (here 128 column pairs x 40 columns) computes each value where it is used.  Both paths go through the
    same checks, and on a geometry that fits the table they are compared with each other through the oracle."""
    w = wl.with_overrides(wl.WORKLOADS["tiny"], name="rope-no-table", heads=2, head_dim=256, grid_h=3, grid_w=90, tile_h=1, tile_w=40)
    run_rope(w, 2, (0, 0, 128), 10000.0, 2)
    run_rope(w, 2, (40, 40, 48), 10000.0, 2)         # 40 + 40 + 48 * 40 = 2000 entries: the table again
