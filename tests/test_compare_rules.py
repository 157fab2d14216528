"""CPU self-tests of the acceptance rules in oracle/compare.py.

The index-set rule is the only thing between a wrong kept set and a green parity report when the
candidate's set differs from the oracle's, so it is exercised here with planted mistakes: each wrong
set must be rejected, and only a swap inside the tie band may pass (and must be counted as a band
case whose sets differ).
"""
import numpy as np
import pytest

from oracle.compare import GAP_REL, check_index_sets, out_tolerance


def _case_with_gap():
    """n = 12, k = 4, a wide gap between the 4th and the 5th largest score."""
    s = np.array([5.0, -1.0, 9.0, 0.5, 7.0, 0.25, 8.0, -3.0, 0.75, 0.1, -0.2, 0.3])
    want = np.array([0, 2, 4, 6], dtype=np.int32)          # 9, 8, 7, 5 | next is 0.75
    return s[None, None, :], 4, want


def _case_with_band():
    """n = 10, k = 3: the 3rd and 4th scores differ by 1e-5 relative (inside the band), a third
    score sits in the band as well, everything else is far away."""
    s = np.array([0.0, 10.0, 4.0, 4.0 * (1 - 1e-5), 9.0, -2.0, 4.0 * (1 - 2e-5), 1.0, 3.0, -7.0])
    want = np.array([1, 2, 4], dtype=np.int32)             # 10, 9, 4.0 | band: rows 2, 3, 6
    return s[None, None, :], 3, want


def _row(sel, k):
    idx = np.full((1, 1, k), -1, dtype=np.int32)
    idx[0, 0, :len(sel)] = sel
    return idx, np.array([[len(sel)]], dtype=np.int32)


def test_the_oracle_set_passes_under_both_rules():
    for s, k, want in (_case_with_gap(), _case_with_band()):
        rep = check_index_sets(s, k, None, *_row(want, k))
        assert rep.ok and rep.equal_sets == 1 and rep.problems == 1
    assert check_index_sets(*_case_with_gap()[:2], None, *_row(_case_with_gap()[2], 4)).exact_rule == 1
    rep = check_index_sets(*_case_with_band()[:2], None, *_row(_case_with_band()[2], 3))
    assert rep.band_rule == 1 and rep.boundary_ties == [3]


def test_a_swap_across_a_wide_gap_is_rejected():
    s, k, want = _case_with_gap()
    wrong = np.array([2, 4, 6, 8], dtype=np.int32)         # 5.0 out, 0.75 in
    rep = check_index_sets(s, k, None, *_row(wrong, k))
    assert not rep.ok and rep.equal_sets == 0 and rep.exact_rule == 1


def test_a_swap_inside_the_band_passes_and_is_counted_as_a_band_case_with_different_sets():
    s, k, want = _case_with_band()
    for other in (3, 6):
        swapped = np.sort(np.array([1, 4, other], dtype=np.int32))
        rep = check_index_sets(s, k, None, *_row(swapped, k))
        assert rep.ok, rep.failures
        assert rep.band_rule == 1 and rep.equal_sets == 0 and rep.boundary_ties == [3]
        assert rep.summary()["boundary_ties_total"] == 3


def test_band_rule_rejects_a_far_token_kept_and_a_top_token_dropped():
    s, k, want = _case_with_band()
    far_in = np.array([1, 4, 8], dtype=np.int32)           # 3.0 is far below the band
    rep = check_index_sets(s, k, None, *_row(far_in, k))
    assert not rep.ok and any("below the tie band" in f for f in rep.failures)
    top_out = np.array([2, 3, 4], dtype=np.int32)          # 10.0 dropped, two band members kept
    rep = check_index_sets(s, k, None, *_row(top_out, k))
    assert not rep.ok and any("above the tie band" in f for f in rep.failures)


def test_band_width_is_the_stated_relative_gap():
    """A gap just above 1e-3 relative is judged exactly, one just below by the band."""
    base = np.array([3.0, 2.0, 1.0, 0.0])
    for rel, exact in ((1.2 * GAP_REL, True), (0.8 * GAP_REL, False)):
        s = base.copy()
        s[2] = 2.0 * (1 - rel)                             # k = 2: 2.0 is the k-th, s[2] the (k+1)-th
        swapped = np.array([0, 2], dtype=np.int32)
        rep = check_index_sets(s[None, None, :], 2, None, *_row(swapped, 2))
        assert rep.exact_rule == int(exact) and rep.band_rule == int(not exact)
        assert rep.ok == (not exact)


@pytest.mark.parametrize("what", ["duplicate", "out_of_range", "negative", "wrong_count", "short_count",
                                  "padding_not_minus_one", "descending"])
def test_malformed_rows_are_rejected(what):
    s, k, want = _case_with_gap()
    idx, cnt = _row(want, k)
    if what == "duplicate":
        idx[0, 0] = [0, 2, 2, 6]
    elif what == "out_of_range":
        idx[0, 0] = [0, 2, 4, 12]
    elif what == "negative":
        idx[0, 0] = [-1, 2, 4, 6]
    elif what == "wrong_count":
        cnt[0, 0] = 5
    elif what == "short_count":
        cnt[0, 0] = 3
        idx[0, 0, 3] = -1
    elif what == "padding_not_minus_one":
        s = s[:, :, :3]                                     # kb = 3 < k: slot 3 must hold -1
        idx[0, 0] = [0, 1, 2, 0]
        cnt[0, 0] = 3
    elif what == "descending":
        idx[0, 0] = [6, 4, 2, 0]
    rep = check_index_sets(s, k, None, idx, cnt)
    assert not rep.ok, what


def test_lengths_ties_and_trivial_sets():
    # vis_len cuts the row: the large score past the length must not be wanted, and keeping it fails
    s = np.array([[[1.0, 2.0, 3.0, 100.0]]])
    vis_len = np.array([3])
    assert check_index_sets(s, 2, vis_len, *_row(np.array([1, 2]), 2)).ok
    assert not check_index_sets(s, 2, vis_len, *_row(np.array([2, 3]), 2)).ok
    # exact ties: the lower index is the oracle's choice; the other member of the tie lies in the band
    t = np.array([[[5.0, 1.0, 5.0, 5.0, 0.0]]])
    rep = check_index_sets(t, 2, None, *_row(np.array([0, 2]), 2))
    assert rep.ok and rep.equal_sets == 1 and rep.band_rule == 1
    rep = check_index_sets(t, 2, None, *_row(np.array([0, 3]), 2))
    assert rep.ok and rep.equal_sets == 0
    # k >= n: everything is kept, anything else fails; k = 0: empty
    full = check_index_sets(t, 7, None, *_row(np.arange(5), 7))
    assert full.ok and full.exact_rule == 1
    assert not check_index_sets(t, 5, None, *_row(np.array([0, 1, 2, 3]), 5)).ok
    assert check_index_sets(t, 0, None, np.zeros((1, 1, 0), np.int32), np.zeros((1, 1), np.int32)).ok
    # several problems: one bad (b, g) is enough to fail, and it is named
    s2 = np.stack([_case_with_gap()[0][0], _case_with_gap()[0][0]], axis=0)      # [2, 1, 12]
    idx = np.stack([_row(_case_with_gap()[2], 4)[0][0], _row(np.array([2, 4, 6, 8]), 4)[0][0]], axis=0)
    cnt = np.array([[4], [4]], dtype=np.int32)
    rep = check_index_sets(s2, 4, None, idx, cnt)
    assert rep.problems == 2 and rep.equal_sets == 1 and len(rep.failures) == 1 and "b=1" in rep.failures[0]


def test_output_tolerances_are_the_stated_ones():
    assert out_tolerance(np.float16) == 2e-3 and out_tolerance(np.float32) == 1e-5
    with pytest.raises(KeyError):
        out_tolerance(np.float64)
