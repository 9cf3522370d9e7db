"""The parity harness's own acceptance rules, checked on the CPU: what counts as a documented
near-tie (relative score gap below 1e-5 between the entries that differ) and what does not."""
import numpy as np

from tests import harness


def _scores():
    #        id:  0     1            2     3      4     5
    return np.array([5.0, 4.0 + 1e-7, 4.0, 1.0, -np.inf, 0.5])


def test_identical_lists_pass():
    assert harness.selection_within_near_ties([0, 1, 2], [0, 1, 2], _scores())


def test_exchange_of_near_tied_neighbours_passes_inside_the_list_and_at_the_cut():
    sc = _scores()
    assert harness.selection_within_near_ties([0, 2, 1], [0, 1, 2], sc)      # inside the list
    assert harness.selection_within_near_ties([0, 2], [0, 1], sc)            # across the k / k+1 cut


def test_a_near_tie_elsewhere_in_the_unit_excuses_nothing():
    sc = _scores()
    # ids 1 and 2 are near-tied, but the lists differ at ids 3 / 5, whose scores are far apart
    assert not harness.selection_within_near_ties([0, 1, 2, 5], [0, 1, 2, 3], sc)
    assert not harness.selection_within_near_ties([1, 0, 2], [0, 1, 2], sc)  # 5.0 against 4.0


def test_invalid_lists_fail():
    sc = _scores()
    assert not harness.selection_within_near_ties([0, 1], [0, 1, 2], sc)     # length
    assert not harness.selection_within_near_ties([0, 2, 2], [0, 1, 2], sc)  # an id twice
    assert not harness.selection_within_near_ties([0, 4, 2], [0, 1, 2], sc)  # an empty cluster
    assert not harness.selection_within_near_ties([0, 9, 2], [0, 1, 2], sc)  # not an id


def test_gap_just_above_the_bar_fails():
    sc = np.array([3.0, 2.0 * (1 + 2e-5), 2.0, 1.0])
    assert not harness.selection_within_near_ties([0, 2, 1], [0, 1, 2], sc)
    sc = np.array([3.0, 2.0 * (1 + 5e-6), 2.0, 1.0])
    assert harness.selection_within_near_ties([0, 2, 1], [0, 1, 2], sc)
