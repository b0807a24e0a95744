"""CPU checks of the comparison rules the GPU parity tests apply where the library may legitimately differ from
the oracle: block selections on near-tied rows and eviction decisions on near-tied groups.  Mistakes are planted
in the candidate under test (a made-up selection or decision), never on the GPU."""
import numpy as np
import pytest
import torch

import oracle
from lcsa_harness import EVICT_NEAR_TIE_REL, NEAR_TIE, check_eviction, check_selection

OG = oracle.Geometry(heads=1, head_dim=8, grid_h=8, grid_w=8, tile_h=4, tile_w=4, q_frames=1, radius_h=-1, radius_w=-1, topk=2)


def _row(scores):
    """One head, query block 0 of a 2x2-tile frame, two visible frames (8 key blocks)."""
    S = np.zeros((1, 4, 8))
    S[0, 0] = scores
    S[0, 1:] = np.arange(8)[None, :]                     # other rows: no ties
    idx, cnt, gap = oracle.select(S, OG, 2)
    return S, idx, cnt, gap


def _as_gpu(idx, cnt):
    return torch.from_numpy(idx.copy()), torch.from_numpy(cnt.copy())


def test_identical_selection_passes_and_counts_near_ties():
    S, idx, cnt, gap = _row([5.0, 4.0, 4.0 - 2e-4, 1, 0, 0, 0, 0])
    _, _, n_diff, n_near = check_selection(*_as_gpu(idx, cnt), idx, cnt, gap, OG, 2, S)
    assert (n_diff, n_near) == (0, 1)


def test_exchange_among_near_tied_blocks_is_accepted():
    S, idx, cnt, gap = _row([5.0, 4.0, 4.0 - 2e-4, 1, 0, 0, 0, 0])
    assert list(idx[0, 0]) == [0, 1]
    got = idx.copy()
    got[0, 0] = [0, 2]                                   # the block 2e-4 below the cut instead of the one at the cut
    _, _, n_diff, _ = check_selection(torch.from_numpy(got), torch.from_numpy(cnt), idx, cnt, gap, OG, 2, S)
    assert n_diff == 1


@pytest.mark.parametrize("bad,why", [
    ([0, 3], "a block far below the cut"),
    ([1, 2], "the clear winner dropped"),
    ([2, 0], "not ascending"),
    ([0, 0], "duplicate"),
    ([0, 9], "outside the visible blocks"),
])
def test_near_tie_row_with_an_inadmissible_exchange_fails(bad, why):
    S, idx, cnt, gap = _row([5.0, 4.0, 4.0 - 2e-4, 1, 0, 0, 0, 0])
    got = idx.copy()
    got[0, 0] = bad
    with pytest.raises(AssertionError):
        check_selection(torch.from_numpy(got), torch.from_numpy(cnt), idx, cnt, gap, OG, 2, S)


def test_difference_on_a_row_with_a_clear_gap_fails():
    S, idx, cnt, gap = _row([5.0, 4.0, 3.0, 1, 0, 0, 0, 0])
    got = idx.copy()
    got[0, 0] = [0, 2]
    with pytest.raises(AssertionError, match="gap"):
        check_selection(torch.from_numpy(got), torch.from_numpy(cnt), idx, cnt, gap, OG, 2, S)


def test_window_is_enforced_on_near_tie_rows():
    og = oracle.Geometry(heads=1, head_dim=8, grid_h=8, grid_w=8, tile_h=4, tile_w=4, q_frames=1, radius_h=0, radius_w=0, topk=1)
    S = np.zeros((1, 4, 8))
    S[0, 0, 0], S[0, 0, 4], S[0, 0, 1] = 1.0, 1.0 - 1e-4, 1.0 - 1e-4        # block 1 ties too but lies outside the window
    idx, cnt, gap = oracle.select(S, og, 2)
    assert list(idx[0, 0]) == [0] and gap[0, 0] < NEAR_TIE
    ok, bad = idx.copy(), idx.copy()
    ok[0, 0], bad[0, 0] = [4], [1]
    check_selection(torch.from_numpy(ok), torch.from_numpy(cnt), idx, cnt, gap, og, 2, S)
    with pytest.raises(AssertionError):
        check_selection(torch.from_numpy(bad), torch.from_numpy(cnt), idx, cnt, gap, og, 2, S)


# ---- eviction decisions -----------------------------------------------------------------------------------------

def test_eviction_same_decision_and_near_tie_exchange():
    imp = np.array([[3.0, 1.0, 1.0 + 0.5 * EVICT_NEAR_TIE_REL, 5.0]])
    assert check_eviction([[1]], [[1]], imp, uniform=False) == 0
    assert check_eviction([[2]], [[1]], imp, uniform=False) == 1      # within the band: accepted, reported


def test_eviction_outside_the_band_or_malformed_fails():
    imp = np.array([[3.0, 1.0, 1.0 + 4 * EVICT_NEAR_TIE_REL, 5.0]])
    with pytest.raises(AssertionError):
        check_eviction([[2]], [[1]], imp, uniform=False)
    with pytest.raises(AssertionError):
        check_eviction([[0]], [[1]], imp, uniform=False)
    with pytest.raises(AssertionError):
        check_eviction([[1, 2]], [[1]], imp, uniform=False)             # wrong count


def test_eviction_exact_ties_go_to_the_older_group():
    imp = np.zeros((2, 4))                                            # a cache that was never scored
    assert check_eviction([[0], [0]], [[0], [0]], imp, uniform=False) == 0
    with pytest.raises(AssertionError, match="tie exactly"):
        check_eviction([[0], [1]], [[0], [0]], imp, uniform=False)


def test_uniform_policy_needs_one_decision_for_all_heads():
    imp = np.array([[1.0, 2.0, 3.0], [1.0, 2.0, 3.0]])
    with pytest.raises(AssertionError, match="uniform"):
        check_eviction([[0], [1]], [[0], [0]], imp, uniform=True)


def test_model_follows_a_given_decision():
    m = oracle.ImportanceCache(capacity_frames=3, tile_t=1, heads=1, uniform=False)
    f = lambda x: np.full((4, 1, 2), float(x), np.float32)
    for i in range(3):
        m.append(f(i), f(i), 1)
    m.set_importance(np.array([[2.0, 1.0, 3.0]]))
    assert m.victims(1) == [[1]]
    m.append(f(3), f(3), 1, victims=[[0]])                            # told to drop the oldest instead
    assert m.birth_order().tolist() == [[1, 2, 3]]
    assert (m.importances() == 0).all()
    with pytest.raises(AssertionError):
        m.append(f(4), f(4), 1, victims=[[0, 1]])                     # one group has to go, not two
