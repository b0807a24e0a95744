"""The entry point that allocates nothing (lcsa_block_importance_static: scratch in a static device array of the
library) against the entry point it is a variant of (lcsa_block_importance: scratch inside the cache's memory),
through the C ABI: two calls in a row, the second on a smaller problem, so that the shared array still holds
the first call's partial sums when the second one runs.  Both run the same kernels in the same order, so the
scores must be the same bits; the oracle's values are compared as well."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from lcsa_harness import IMPORTANCE_RTOL, Pipeline, say
from paper_2510_12747_amd import binding as B
from paper_2510_12747_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _scores_both_ways(w, chunks):
    p = Pipeline(w)
    for _ in range(chunks):
        q, qd = p.feed()
    g = p.g
    pq = B.lcsa_pool_blocks(g, qd, g.q_frames)
    gc = g.c()
    L = B.lib()
    stream = torch.cuda.current_stream().cuda_stream
    imp_view = B.lcsa_cache_importance(p.cache)
    imp_view.fill_(-1.0)
    assert L.lcsa_block_importance(ctypes.byref(gc), pq.data_ptr(), p.cache.handle, 0.0, stream) == 0
    want = imp_view.clone()
    imp_view.fill_(-1.0)
    assert L.lcsa_block_importance_static(ctypes.byref(gc), pq.data_ptr(), p.cache.handle, 0.0, stream) == 0
    torch.cuda.synchronize()
    got = imp_view.clone()
    assert torch.equal(got, want), "static-scratch variant differs from lcsa_block_importance"
    kvf = p.model.valid_frames
    K, _ = p.model.visible()
    S = oracle.scores(oracle.pool(q, p.og, g.q_frames), oracle.pool(K, p.og, kvf))
    ref = oracle.group_importance(S, p.og, kvf)
    np.testing.assert_allclose(got.cpu().numpy()[:, :kvf // g.tile_t], ref, rtol=IMPORTANCE_RTOL, atol=1e-5)
    return got


def test_static_scratch_variant_matches_on_two_calls_the_second_smaller():
    say("no-alloc entry point: small-video shape (12 heads, 18 query blocks, 3 groups)")
    _scores_both_ways(wl.WORKLOADS["small"], 3)
    say("no-alloc entry point: smaller problem right after (2 heads, 9 query blocks, 2 of 4 groups visible)")
    _scores_both_ways(wl.with_overrides(wl.WORKLOADS["small"], name="noalloc-small", heads=2, q_frames=1, cache_frames=4), 2)


def test_static_scratch_variant_rejects_what_does_not_fit():
    """heads * n_qb * groups beyond the array: refused on the host with a clear status, nothing is launched
    (the caches here are handles over an address that is never touched)."""
    fits = B.Geom(64, 128, 512, 512, 8, 16, 1, 2, 24, 24, 32)       # 64 heads x 2048 query blocks x 2 groups = 262144 floats
    big = B.Geom(64, 128, 512, 512, 8, 16, 1, 3, 24, 24, 32)        # x 3 groups: beyond the array
    L = B.lib()
    for geom, want in ((fits, -1), (big, -2)):                      # -1: only the empty cache is at fault; -2: unsupported
        h = ctypes.c_void_p()
        gc = geom.c()
        assert L.lcsa_cache_init(ctypes.byref(h), ctypes.byref(gc), ctypes.c_void_p(1 << 20), B.lcsa_cache_device_bytes(geom)) == 0
        assert L.lcsa_block_importance_static(ctypes.byref(gc), ctypes.c_void_p(1 << 20), h, 0.0, None) == want
        L.lcsa_cache_free(h)
    assert "unsupported" in B.lcsa_status_string(-2)
