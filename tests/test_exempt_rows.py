"""The validity rule for mask rows that are exempt from bit-exactness (near ties; Sec. 3.2 eq. 8):
the check used by the GPU parity tests must accept every row a correct kernel can produce and
reject rows that merely have the right count.  Runs on the CPU, on hand-built rows."""
import numpy as np
import pytest

from oracle import rf2_oracle as orc
from tests import helpers as hp


def _row(scores):
    S = np.array([scores], dtype=np.float64)
    sink_cols = np.zeros(S.shape[1], dtype=bool)
    return S, sink_cols


def test_top_n_row_may_only_trade_columns_inside_the_tie():
    # k_sel = 2: scores 5, 3.0004, 3.0000, 1 -> columns 1 and 2 are 4e-4 apart (a near tie), column 3 is far
    S, sink_cols = _row([5.0, 3.0004, 3.0, 1.0])
    M_ref = orc.select_blocks(S, 2, 0, 0)
    assert orc.selection_gap(S, 2, 0, 0)[0] <= hp.TIE_GAP
    exempt = np.array([True])
    same = M_ref.copy()
    assert hp.check_exempt_rows(same, M_ref, S, exempt, sink_cols, k_sel=2) == 0
    swapped = np.array([[True, False, True, False]])                 # took the other member of the tie
    assert hp.check_exempt_rows(swapped, M_ref, S, exempt, sink_cols, k_sel=2) == 1
    with pytest.raises(AssertionError):                              # right count, but a column far below the boundary
        hp.check_exempt_rows(np.array([[True, False, False, True]]), M_ref, S, exempt, sink_cols, k_sel=2)
    with pytest.raises(AssertionError):                              # dropped the clear winner
        hp.check_exempt_rows(np.array([[False, True, True, False]]), M_ref, S, exempt, sink_cols, k_sel=2)
    with pytest.raises(AssertionError):                              # wrong count
        hp.check_exempt_rows(np.array([[True, True, True, False]]), M_ref, S, exempt, sink_cols, k_sel=2)


def test_top_n_row_must_keep_the_sink_columns():
    S = np.array([[5.0, 3.0004, 3.0, 1.0, 0.0]])
    sink_cols = np.array([False, False, False, False, True])
    M_ref = orc.select_blocks(S, 2, 5, 5, (4, 5))
    got = M_ref.copy()
    got[0, 4] = False
    with pytest.raises(AssertionError):
        hp.check_exempt_rows(got, M_ref, S, np.array([True]), sink_cols, k_sel=2)


def test_cumulative_mass_row_is_a_prefix_cut_at_most_one_column_off():
    d = 4
    S = 2.0 * np.log(np.array([[0.4, 0.3, 0.2, 0.1]]))              # cumulative 0.4, 0.7, 0.9, 1.0
    sink_cols = np.zeros(4, dtype=bool)
    M_ref, margin = orc.select_blocks_cdf(S, 0.7, d, 0, 0)           # cut exactly on 0.7: two columns, margin ~0
    assert M_ref[0].tolist() == [True, True, False, False] and margin[0] < hp.CDF_TIE
    ex = np.array([True])
    assert hp.check_exempt_rows(M_ref.copy(), M_ref, S, ex, sink_cols, d=d) == 0
    assert hp.check_exempt_rows(np.array([[True, True, True, False]]), M_ref, S, ex, sink_cols, d=d) == 1   # one later
    assert hp.check_exempt_rows(np.array([[True, False, False, False]]), M_ref, S, ex, sink_cols, d=d) == 1  # one earlier
    with pytest.raises(AssertionError):                              # two columns off
        hp.check_exempt_rows(np.array([[True, True, True, True]]), M_ref, S, ex, sink_cols, d=d)
    with pytest.raises(AssertionError):                              # right length, not a prefix of the descending order
        hp.check_exempt_rows(np.array([[True, False, True, False]]), M_ref, S, ex, sink_cols, d=d)
    with pytest.raises(AssertionError):                              # empty row
        hp.check_exempt_rows(np.array([[False, False, False, False]]), M_ref, S, ex, sink_cols, d=d)


def test_rows_that_are_not_exempt_are_not_looked_at():
    S, sink_cols = _row([5.0, 3.0004, 3.0, 1.0])
    M_ref = orc.select_blocks(S, 2, 0, 0)
    assert hp.check_exempt_rows(~M_ref, M_ref, S, np.array([False]), sink_cols, k_sel=2) == 0
