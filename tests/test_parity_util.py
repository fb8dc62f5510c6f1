"""The comparison helpers of the GPU parity tests, exercised on the CPU: the oracle's own table stands in for
the library's, and mistakes are planted in that copy.  Every planted mistake must be caught, in entries that
are compared exactly and in entries that a near-tie excuses from the exact comparison."""
import numpy as np
import pytest

import oracle
import parity_util
import skim_synth


@pytest.fixture(scope="module")
def table():
    W, S = skim_synth.make_ws_small(4242, 12, 300, zero_s_frac=0.2)
    S[5] = 0.0                                        # a row clustered with unit weights
    ref = oracle.error_table(W, S, count_near=True)
    ref["near_rb"][:] = 0
    ref["near_rb"][3, 2] = 1                          # pretend the oracle met a near-tie in these entries
    ref["near_rb"][5, 3] = 2
    ref["near_rb"][7, 0] = 1
    return W, S, ref


def copy_of(ref):
    return ref["E"].copy(), ref["centroids_all"].copy(), ref["upper_all"].copy()


def test_the_oracles_own_table_passes(table):
    W, S, ref = table
    E, ca, ua = copy_of(ref)
    st = parity_util.compare_table(W, S, None, ref, E, ca, ua)
    assert st["excused"] == 3 and st["differ"] == 0


OFF = {1: 0, 2: 2, 3: 6, 4: 14}


@pytest.mark.parametrize("row,b", [(0, 1), (3, 3), (5, 4), (7, 1), (11, 4)])
def test_planted_mistakes_are_caught_in_clean_and_in_excused_entries(table, row, b):
    W, S, ref = table
    K = 1 << b
    sl = slice(OFF[b], OFF[b] + K)
    # an error off by 1e-4 relative
    E, ca, ua = copy_of(ref)
    E[row, b - 1] *= 1 + 1e-4
    with pytest.raises(AssertionError):
        parity_util.compare_table(W, S, None, ref, E, ca, ua)
    # a centroid off by 1e-4 relative (one that has members with mass)
    E, ca, ua = copy_of(ref)
    k = int(np.argmax(np.isfinite(ua[row, sl]) & (np.abs(ca[row, sl]) > 1e-3)))
    ca[row, OFF[b] + k] *= 1 + 1e-4
    with pytest.raises(AssertionError):
        parity_util.compare_table(W, S, None, ref, E, ca, ua)
    # a threshold moved to the next smaller value of the row: one element changes cluster
    E, ca, ua = copy_of(ref)
    fin = np.flatnonzero(np.isfinite(ua[row, sl]))
    k = fin[np.argsort(ua[row, sl][fin])[0]]         # lowest cluster with members
    vals = np.unique(W[row].astype(np.float64))
    below = vals[vals < ua[row, OFF[b] + k]]
    if len(below) and K > 1 and len(fin) > 1:
        ua[row, OFF[b] + k] = below[-1]
        with pytest.raises(AssertionError):
            parity_util.compare_table(W, S, None, ref, E, ca, ua)
    # a threshold that is no value of the row
    E, ca, ua = copy_of(ref)
    ua[row, OFF[b] + fin[0]] += 1e-6
    with pytest.raises(AssertionError):
        parity_util.compare_table(W, S, None, ref, E, ca, ua)


def test_row_self_consistency_catches_a_flipped_label():
    W, S = skim_synth.make_ws_small(99, 6, 200)
    bits = np.array([1, 2, 3, 4, 2, 3], np.uint8)
    rr = oracle.cluster_rows(W, S, bits)
    parity_util.check_rows_self_consistent(W, S, None, bits, rr["labels"], rr["centroids"], rr["upper"], rr["err"])
    lab = rr["labels"].copy()
    lab[3, 17] ^= 1
    with pytest.raises(AssertionError):
        parity_util.check_rows_self_consistent(W, S, None, bits, lab, rr["centroids"], rr["upper"], rr["err"])
    al = skim_synth.make_alpha(1, 200, spread=0.2)
    ra = oracle.cluster_rows(W, S, bits, alpha=al)
    parity_util.check_rows_self_consistent(W, S, al, bits, ra["labels"], ra["centroids"], ra["upper"], ra["err"])
    with pytest.raises(AssertionError):      # the unscaled clustering is not a clustering of the scaled rows
        parity_util.check_rows_self_consistent(W, S, al, bits, rr["labels"], rr["centroids"], rr["upper"], rr["err"])
