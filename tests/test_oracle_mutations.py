"""The pins must be able to fail: each case below plants ONE plausible mistake in the oracle (on the
CPU, by wrapping the oracle's own function) and checks that at least one of the pin tests then fails.
A mistake no pin notices would mean that part of the oracle is unpinned."""
import numpy as np
import pytest

from oracle import rf2_oracle as orc
from tests import test_oracle_attention as t_attn
from tests import test_oracle_mask as t_mask
from tests import test_oracle_perm as t_perm

REAL = {n: getattr(orc, n) for n in ("perm_table", "inverse_table", "unpermute", "sink_block_range", "budget",
                                     "pool_blocks", "block_scores", "select_blocks", "select_blocks_cdf",
                                     "block_sparse_attention", "selection_gap", "kept_pairs", "default_window")}


def _perm_sink_front(*a, **k):                      # ignores "first frame moved to the end"
    a = list(a)
    if len(a) > 7:
        a[7] = False
    else:
        k["sink_at_end"] = False
    return REAL["perm_table"](*a, **k)


def _perm_hw_swapped(T, H, W, wt, wh, ww, *a, **k):  # windows over (w, h) instead of (h, w)
    p = REAL["perm_table"](T, W, H, wt, ww, wh, *a, **k)
    n_video = T * H * W
    out = p.copy()
    v = p < n_video
    t, h, w = p[v] // (H * W), (p[v] // H) % W, p[v] % H          # decode in the transposed grid
    out[v] = (t * H + w) * W + h
    return out


def _pool_divides_by_b(Xp, b):                      # ragged block averaged over b rows instead of its own
    m = REAL["pool_blocks"](Xp, b).copy()
    last = Xp.shape[0] - (m.shape[0] - 1) * b
    m[-1] *= last / b
    return m


def _select_drops_sink_columns(S, k_sel, sb, se, sink_k=None):
    M = REAL["select_blocks"](S, k_sel, sb, se, sink_k).copy()
    kb, ke = (sb, se) if sink_k is None else sink_k
    rows = np.ones(M.shape[0], dtype=bool)
    rows[sb:se] = False
    M[np.ix_(rows, np.arange(kb, ke))] = False
    return M


def _select_ties_prefer_higher_column(S, k_sel, sb, se, sink_k=None):
    M = REAL["select_blocks"](S[:, ::-1], k_sel, sb, se, None if sink_k is None else sink_k)
    return M[:, ::-1] if sb == se else REAL["select_blocks"](S + np.arange(S.shape[1]) * 1e-300, k_sel, sb, se, sink_k)


def _select_sink_rows_not_dense(S, k_sel, sb, se, sink_k=None):
    M = REAL["select_blocks"](S, k_sel, sb, se, sink_k).copy()
    M[sb:se, :1] = False
    return M


def _attn_without_scaling(Qp, Kp, *a, **k):          # drops the 1/sqrt(d) of eq. (1)
    return REAL["block_sparse_attention"](Qp * np.sqrt(np.sqrt(Qp.shape[1])), Kp * np.sqrt(np.sqrt(Qp.shape[1])), *a, **k)


def _attn_transposed_mask(Qp, Kp, Vp, M, *a, **k):   # skip rule applied to M[j, i]
    return REAL["block_sparse_attention"](Qp, Kp, Vp, M.T.copy() if M.shape[0] == M.shape[1] else M, *a, **k)


def _attn_uses_k_for_v(Qp, Kp, Vp, *a, **k):
    return REAL["block_sparse_attention"](Qp, Kp, Kp[:, :Vp.shape[1]] if Kp.shape[1] >= Vp.shape[1] else Vp, *a, **k)


def _attn_wrong_normaliser(*a, **k):                 # final division of eq. (4) slightly off
    r = REAL["block_sparse_attention"](*a, **k)
    return (r[0] * 0.999, r[1]) if isinstance(r, tuple) else r * 0.999


def _budget_ceil(*a, **k):
    kr, ks = REAL["budget"](*a, **k)
    return (kr + 1, ks + 1)


def _sink_range_misses_straddling_block(N, frame, b, sf, at_end=True, text=0):
    lo, hi = REAL["sink_block_range"](N, frame, b, sf, at_end, text)
    if hi > lo and at_end and (N - sf * frame - text) % b:
        lo += 1                                      # ceil instead of floor: drops the block holding both kinds
    return (lo, hi)


def _cdf_normalises_over_all_columns(S, tau, d, sb, se, sink_k=None):
    return REAL["select_blocks_cdf"](S, tau, d, sb, sb, (se, se) if sink_k is None else (sink_k[1], sink_k[1]))


def _cdf_forgets_sqrt_d(S, tau, d, *a, **k):
    return REAL["select_blocks_cdf"](S, tau, 1, *a, **k)


def _cdf_margin_one_sided(side):
    """The margin computed from one side of the cut only (the other side forgotten)."""
    def mutant(S, tau, d, sb, se, sink_k=None):
        M, margin = REAL["select_blocks_cdf"](S, tau, d, sb, se, sink_k)
        kb, ke = (sb, se) if sink_k is None else sink_k
        cand = np.array([j for j in range(S.shape[1]) if not (kb <= j < ke)])
        for i in np.flatnonzero(np.isfinite(margin)):
            p = np.exp((S[i, cand] - S[i, cand].max()) / np.sqrt(d))
            cum = np.cumsum(np.sort(p / p.sum())[::-1])
            n = int(M[i, cand].sum())
            margin[i] = abs(cum[n - 1] - tau) if side == "after" else abs(tau - (cum[n - 2] if n >= 2 else 0.0))
        return M, margin
    return mutant


def _window_256_keeps_the_128_shape(block, video):
    return REAL["default_window"](min(block, 128), video)


def _call_all(tests):
    """Runs pin tests (plain functions, with their parameter sets); returns True if any of them fails."""
    for fn, argsets in tests:
        for args in argsets:
            try:
                fn(*args)
            except AssertionError:
                return True
            except Exception:                         # a mutant may also crash a pin: counts as noticed
                return True
    return False


PERM_ROWS = [(r,) for r in t_perm._rows("perm_examples.txt")]
SIZE_ROWS = [(r,) for r in t_perm._rows("config_sizes.txt")]
RECT_ROWS = [(r,) for r in t_perm._rows("config_sizes_rect.txt")]

MUTANTS = {
    "perm: sink left at the front": ("perm_table", _perm_sink_front, [(t_perm.test_perm_matches_hand_written_examples, PERM_ROWS)]),
    "perm: window axes swapped": ("perm_table", _perm_hw_swapped, [(t_perm.test_perm_matches_hand_written_examples, PERM_ROWS)]),
    "inverse table = forward table": ("inverse_table", lambda p: p.copy(), [(t_perm.test_round_trip_is_identity, [()]),
                                                                              (t_attn.test_layer_sparse_equals_library_attention_in_raster_order, [()])]),
    "unpermute gathers instead of scatters": ("unpermute", lambda Xp, perm: Xp[perm], [(t_perm.test_round_trip_is_identity, [()])]),
    "sink range drops the straddling block": ("sink_block_range", _sink_range_misses_straddling_block,
                                              [(t_perm.test_sink_block_range_front_and_straddle, [()]), (t_perm.test_sizes_of_the_workloads, SIZE_ROWS)]),
    "budget off by one": ("budget", _budget_ceil, [(t_perm.test_sizes_of_the_workloads, SIZE_ROWS),
                                                   (t_perm.test_sizes_with_different_q_and_k_blocks, RECT_ROWS)]),
    "ragged block mean divides by b": ("pool_blocks", _pool_divides_by_b, [(t_mask.test_pool_constant_block_and_weighted_sum, [()])]),
    "scores scaled by 1/sqrt(d) (eq. 7 has no scale)": ("block_scores", lambda q, k: REAL["block_scores"](q, k) / np.sqrt(q.shape[1]),
                                                        [(t_mask.test_scores_definition_by_loops, [()])]),
    "selection forgets the sink columns": ("select_blocks", _select_drops_sink_columns,
                                           [(t_mask.test_select_vs_brute_force, [(12, 9, 12, 3), (9, 0, 3, 2)])]),
    "ties prefer the higher column": ("select_blocks", _select_ties_prefer_higher_column, [(t_mask.test_ties_prefer_lower_column, [()])]),
    "sink rows not dense": ("select_blocks", _select_sink_rows_not_dense, [(t_mask.test_select_vs_brute_force, [(12, 9, 12, 3)])]),
    "attention without 1/sqrt(d)": ("block_sparse_attention", _attn_without_scaling, [(t_attn.test_all_blocks_kept_equals_dense_attention, [()])]),
    "skip rule on the transposed mask": ("block_sparse_attention", _attn_transposed_mask,
                                         [(t_attn.test_masked_equals_library_masked_attention, [(256, 64, 0.5), (200, 32, 0.4)])]),
    "values taken from K": ("block_sparse_attention", _attn_uses_k_for_v, [(t_attn.test_all_blocks_kept_equals_dense_attention, [()])]),
    "wrong final normaliser": ("block_sparse_attention", _attn_wrong_normaliser, [(t_attn.test_constant_and_one_hot_values, [()])]),
    "cdf normalises over sink columns too": ("select_blocks_cdf", _cdf_normalises_over_all_columns,
                                             [(t_mask.test_cdf_selection_vs_loops, [(12, 9, 12, 0.5), (17, 14, 17, 0.97)])]),
    "cdf margin looks only after the cut": ("select_blocks_cdf", _cdf_margin_one_sided("after"), [(t_mask.test_cdf_margin_by_hand, [()])]),
    "cdf margin looks only before the cut": ("select_blocks_cdf", _cdf_margin_one_sided("before"), [(t_mask.test_cdf_margin_by_hand, [()])]),
    "256-token blocks get the 128-token window": ("default_window", _window_256_keeps_the_128_shape,
                                                  [(t_perm.test_interior_window_is_one_block, [()])]),
    "cdf forgets 1/sqrt(d)": ("select_blocks_cdf", _cdf_forgets_sqrt_d, [(t_mask.test_cdf_selection_vs_loops, [(12, 9, 12, 0.5), (12, 0, 0, 0.9)])]),
}


@pytest.mark.parametrize("name", list(MUTANTS))
def test_a_planted_mistake_is_noticed(name, monkeypatch):
    target, mutant, pins = MUTANTS[name]
    assert not _call_all(pins), "the pins must pass on the real oracle"
    monkeypatch.setattr(orc, target, mutant)
    assert _call_all(pins), f"no pin noticed: {name}"
