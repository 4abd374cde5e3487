"""The comparison helpers of the GPU tests, checked on the host: a rule that cannot fail proves nothing."""
import numpy as np
import pytest

import synth_inputs as syn
from helpers import assert_close_max, assert_gate_close, check_routing_against_fp64, own_logits_selection


@pytest.mark.parametrize("k,renorm", [(1, False), (2, False), (2, True)])
def test_own_logits_selection_is_the_oracle_rule(oracle, k, renorm):
    g = syn.rng(900 + k)
    logits = g.standard_normal((300, 17)).astype(np.float32)
    logits[::3] = np.round(logits[::3])  # exact ties: the lowest id wins on both sides
    idx, w = own_logits_selection(logits, k, renorm)
    idx_ref, w_ref = oracle.topk(logits.astype(np.float64), k, renorm)
    np.testing.assert_array_equal(idx, idx_ref)
    np.testing.assert_allclose(w, w_ref, rtol=1e-12)


def test_assert_close_max_rejects_what_it_should():
    g = syn.rng(901)
    ref = g.standard_normal((40, 64))
    ref[5] = 0.0  # a token without a kept assignment
    assert_close_max(ref * (1 + 1e-3), ref, 2e-2, "scaled")
    bad = ref.copy()
    bad[5, 3] = 1e-3  # a zero row must stay zero
    with pytest.raises(AssertionError):
        assert_close_max(bad, ref, 2e-2, "zero row touched")
    bad = ref.copy()
    bad[7] *= 1.5  # one wrong row, far below the largest element of the matrix
    bad[7] *= 0.01 / np.abs(ref).max()
    ref2 = ref.copy()
    ref2[7] *= 0.01 / np.abs(ref).max()
    with pytest.raises(AssertionError):
        assert_close_max(bad, ref2, 2e-2, "small row wrong by half")
    with pytest.raises(AssertionError):
        assert_close_max(ref[:, ::-1], ref, 2e-2, "columns reversed")
    # a token whose two large expert outputs cancel: the error of the sum is relative to the summands
    a = g.standard_normal((40, 64))
    b = g.standard_normal((40, 64))
    a[0], b[0] = 3.0, -2.99
    got = a * (1 + 2.0 ** -9) + b
    with pytest.raises(AssertionError):
        assert_close_max(got, a + b, 2e-2, "cancellation without the magnitudes")
    assert_close_max(got, a + b, 2e-2, "cancellation", mag=np.abs(a) + np.abs(b))


def test_routing_check_separates_clear_and_near_tied_tokens():
    logits = np.array([[0.0, 1.0, 3.0], [2.0, 2.0 + 1e-7, -1.0], [5.0, 4.0, 3.0]])
    assert check_routing_against_fp64(np.array([[2], [0], [0]]), logits, 1, 1e-4) == 1  # the near-tie may go either way
    assert check_routing_against_fp64(np.array([[2], [1], [0]]), logits, 1, 1e-4) == 1
    with pytest.raises(AssertionError):
        check_routing_against_fp64(np.array([[1], [0], [0]]), logits, 1, 1e-4)  # a clear token decided wrongly
    with pytest.raises(AssertionError):
        check_routing_against_fp64(np.array([[2], [2], [0]]), logits, 1, 1e-4)  # a near-tie resolved to a far expert
    with pytest.raises(AssertionError):
        assert_gate_close(np.array([1.0002]), np.array([1.0]), 1e-4)


def test_stratified_sample_reaches_every_row_tile():
    """Every aligned block of 64 rows of every expert holds a sampled row, so does every coarser
    row tile (256-row tiles, 64-row remainder tiles, a masked last tile), however ragged the loads."""
    from helpers import STRATUM_ROWS, sample_rows, strata_covered

    g = syn.rng(902)
    counts = np.concatenate([[0, 1, 63, 64, 65, 255, 256, 257, 4649], g.integers(0, 700, size=23)])
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    rows = sample_rows(offsets, 1, 7)
    n, hit = strata_covered(offsets, rows)
    assert hit == n == sum(-(-int(c) // STRATUM_ROWS) for c in counts)
    assert (np.diff(rows) > 0).all() and rows.min() >= 0 and rows.max() < offsets[-1]
    for e, c in enumerate(counts):  # first and last row of every non-empty expert
        if c:
            assert offsets[e] in rows and offsets[e + 1] - 1 in rows
    for tile in (64, 128, 256):  # coarser tiles counted from the expert's first row
        for e, c in enumerate(counts):
            mine = rows[(rows >= offsets[e]) & (rows < offsets[e + 1])] - offsets[e]
            assert len(np.unique(mine // tile)) == -(-int(c) // tile)
    big = sample_rows(offsets, 1, 7, min_rows=1024)
    assert len(big) >= 1024 and strata_covered(offsets, big) == (n, n)
    assert len(sample_rows(np.array([0, 5, 5, 9]), 1, 3, min_rows=1024)) == 9  # never more rows than there are
    # a sample that misses a block is reported as such
    assert strata_covered(offsets, rows[rows >= 64])[1] < n
