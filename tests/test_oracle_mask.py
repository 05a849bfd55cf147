"""Pins for the oracle's pooling, scoring and block selection (CPU only)."""
import numpy as np
import pytest

from oracle import rf2_oracle as orc


def test_pool_constant_block_and_weighted_sum():
    rng = np.random.default_rng(1)
    N, d, b = 300, 8, 64                       # last block has 44 rows
    X = rng.standard_normal((N, d))
    X[64:128] = X[64]                          # a block of identical rows
    m = orc.pool_blocks(X, b)
    assert m.shape == (5, d)
    assert np.abs(m[1] - X[64]).max() < 1e-14
    cnt = np.array([64, 64, 64, 64, 44])[:, None]
    assert np.allclose((m * cnt).sum(0), X.sum(0), rtol=0, atol=1e-11)
    assert np.allclose(m[4], X[256:].sum(0) / 44, rtol=0, atol=1e-14)   # ragged block: own count


def test_scores_definition_by_loops():
    rng = np.random.default_rng(2)
    q, k = rng.standard_normal((5, 7)), rng.standard_normal((6, 7))
    S = orc.block_scores(q, k)
    for i in range(5):
        for j in range(6):
            assert abs(S[i, j] - sum(q[i, c] * k[j, c] for c in range(7))) < 1e-13
    assert np.allclose(orc.block_scores(q, q), orc.block_scores(q, q).T)


def brute_force_select(S, k_sel, sb, se):
    """Repeatedly take the maximum (first occurrence) among remaining non-sink columns."""
    Tb = S.shape[0]
    M = np.zeros((Tb, Tb), dtype=bool)
    for i in range(Tb):
        if sb <= i < se:
            M[i] = True
            continue
        left = [j for j in range(Tb) if not (sb <= j < se)]
        for _ in range(k_sel):
            best = left[0]
            for j in left:
                if S[i, j] > S[i, best]:
                    best = j
            M[i, best] = True
            left.remove(best)
        M[i, sb:se] = True
    return M


@pytest.mark.parametrize("Tb,sb,se,k_sel", [(12, 9, 12, 3), (12, 0, 0, 5), (12, 0, 2, 4), (7, 5, 7, 0), (9, 0, 0, 9)])
def test_select_vs_brute_force(Tb, sb, se, k_sel):
    rng = np.random.default_rng(Tb * 100 + k_sel)
    S = rng.standard_normal((Tb, Tb))
    S[1, :] = np.round(S[1, :])                # many exact ties in one row
    M = orc.select_blocks(S, k_sel, sb, se)
    assert np.array_equal(M, brute_force_select(S, k_sel, sb, se))
    for i in range(Tb):
        if sb <= i < se:
            assert M[i].all()
        else:
            assert M[i].sum() == k_sel + (se - sb) and M[i, sb:se].all()
            cand = np.array([j for j in range(Tb) if not (sb <= j < se)])
            kept, dropped = S[i, cand][M[i, cand]], S[i, cand][~M[i, cand]]
            if kept.size and dropped.size:
                assert kept.min() >= dropped.max()


def test_ties_prefer_lower_column():
    S = np.array([[1.0, 3.0, 3.0, 3.0, 0.0],
                  [2.0, 2.0, 2.0, 2.0, 2.0]])
    S = np.vstack([S, np.zeros((3, 5))])
    M = orc.select_blocks(S, 2, 0, 0)
    assert M[0].tolist() == [False, True, True, False, False]
    assert M[1].tolist() == [True, True, False, False, False]


def test_sparsity_zero_keeps_all_and_invariances():
    rng = np.random.default_rng(3)
    N, d, b = 640, 16, 64
    Q, K = rng.standard_normal((N, d)), rng.standard_normal((N, d))
    Tb = orc.n_blocks(N, b)
    k_row, k_sel = orc.budget(Tb, 2, 0.0)
    S = orc.block_scores(orc.pool_blocks(Q, b), orc.pool_blocks(K, b))
    assert orc.select_blocks(S, k_sel, 8, 10).all()
    k_row, k_sel = orc.budget(Tb, 2, 0.5)
    M = orc.select_blocks(S, k_sel, 8, 10)
    # shuffling tokens inside blocks, or scaling Q by a positive constant, cannot change the mask
    Q2, K2 = Q.copy(), K.copy()
    for i in range(Tb):
        Q2[i * b:(i + 1) * b] = Q[i * b:(i + 1) * b][rng.permutation(b)]
        K2[i * b:(i + 1) * b] = K[i * b:(i + 1) * b][rng.permutation(b)]
    S2 = orc.block_scores(orc.pool_blocks(Q2, b), orc.pool_blocks(K2, b))
    assert np.array_equal(orc.select_blocks(S2, k_sel, 8, 10), M)
    assert np.array_equal(orc.select_blocks(4.0 * S, k_sel, 8, 10), M)


def test_selection_gap():
    S = np.array([[5.0, 1.0, 4.0, 3.999, 9.0],
                  [1.0, 2.0, 3.0, 4.0, 9.0],
                  [0.0, 0.0, 0.0, 0.0, 0.0],
                  [0.0, 0.0, 0.0, 0.0, 0.0],
                  [7.0, 7.0, 7.0, 7.0, 7.0]])
    gap = orc.selection_gap(S, 2, 4, 5)        # column/row 4 is the sink
    assert abs(gap[0] - 0.001) < 1e-12 and gap[1] == 1.0 and gap[2] == 0.0 and np.isinf(gap[4])
    assert np.isinf(orc.selection_gap(S, 4, 4, 5)).all()       # every candidate kept: no boundary


def test_mask_to_lists():
    M = np.array([[1, 0, 1], [0, 0, 1], [1, 1, 1]], dtype=bool)
    assert [l.tolist() for l in orc.mask_to_lists(M)] == [[0, 2], [2], [0, 1, 2]]


def _cdf_by_loops(S, tau, d, sb, se):
    """Independent statement of the cumulative-mass rule with explicit loops."""
    Tb = S.shape[0]
    M = np.zeros((Tb, Tb), dtype=bool)
    for i in range(Tb):
        if sb <= i < se:
            M[i] = True
            continue
        cols = [j for j in range(Tb) if not (sb <= j < se)]
        w = {j: np.exp(S[i, j] / np.sqrt(d)) for j in cols}
        total = sum(w.values())
        taken, mass = [], 0.0
        while cols and (not taken or mass < tau * total):
            best = max(cols, key=lambda j: (S[i, j], -j))        # largest score, then lowest column
            cols.remove(best)
            taken.append(best)
            mass += w[best]
        M[i, taken] = True
        M[i, sb:se] = True
    return M


@pytest.mark.parametrize("Tb,sb,se,tau", [(12, 9, 12, 0.5), (12, 0, 0, 0.9), (9, 0, 3, 0.3), (17, 14, 17, 0.97)])
def test_cdf_selection_vs_loops(Tb, sb, se, tau):
    rng = np.random.default_rng(Tb * 7 + int(tau * 100))
    S = rng.standard_normal((Tb, Tb)) * 6.0
    M, margin = orc.select_blocks_cdf(S, tau, 16, sb, se)
    assert np.array_equal(M, _cdf_by_loops(S, tau, 16, sb, se))
    assert M[:, sb:se].all() and M[sb:se].all()
    assert (margin[sb:se] == np.inf).all() and (margin >= 0).all()


def test_cdf_selection_closed_cases():
    Tb, d = 10, 4
    S = np.zeros((Tb, Tb))                                  # equal scores: each of the 8 candidates has mass 1/8
    M, margin = orc.select_blocks_cdf(S, 0.5, d, 8, 10)
    assert (M[:8, :8].sum(1) == 4).all() and M[0, :4].all()  # 4 * 1/8 reaches 0.5; lowest columns first
    assert np.allclose(margin[:8], 0.0)                      # cut exactly on the threshold: flagged as a near-tie
    M, _ = orc.select_blocks_cdf(S, 0.51, d, 8, 10)
    assert (M[:8, :8].sum(1) == 5).all()
    # one dominant column: it alone carries the mass for any tau below its probability
    S = np.zeros((Tb, Tb)); S[:, 3] = 40.0
    M, _ = orc.select_blocks_cdf(S, 0.99, d, 8, 10)
    assert (M[:8, :8].sum(1) == 1).all() and M[:8, 3].all()
    # a larger tau keeps a superset; tau close to 1 keeps (nearly) everything
    rng = np.random.default_rng(3)
    S = rng.standard_normal((Tb, Tb)) * 3.0
    prev = None
    for tau in (0.1, 0.4, 0.7, 0.95, 0.999999):
        M, _ = orc.select_blocks_cdf(S, tau, d, 8, 10)
        assert prev is None or (M | ~prev).all()
        prev = M
    assert prev[:8, :8].sum() >= 8 * 7
    with pytest.raises(ValueError):
        orc.select_blocks_cdf(S, 1.0, d, 8, 10)


def test_cdf_margin_by_hand():
    """Block probabilities 0.4, 0.3, 0.2, 0.1 (scores 2 ln p with d = 4): cumulative 0.4, 0.7, 0.9, 1.
    The margin is the distance from tau to the nearer of the cumulative values just before and just
    after the last column taken; each side decides in one of the cases below."""
    S = 2.0 * np.log(np.array([[0.2, 0.4, 0.1, 0.3]]))       # descending order: columns 1, 3, 0, 2
    for tau, kept, margin in ((0.75, [1, 3, 0], 0.05),       # 0.7 < tau <= 0.9: the side before the cut (0.75 - 0.7)
                              (0.65, [1, 3], 0.05),          # 0.4 < tau <= 0.7: the side after it (0.7 - 0.65)
                              (0.85, [1, 3, 0], 0.05),       # after: 0.9 - 0.85 (before: 0.15)
                              (0.45, [1, 3], 0.05),          # before: 0.45 - 0.4 (after: 0.25)
                              (0.05, [1], 0.05),             # one column: before = the empty sum 0
                              (0.39, [1], 0.01)):            # one column, after: 0.4 - 0.39
        M, m = orc.select_blocks_cdf(S, tau, 4, 0, 0)
        assert np.flatnonzero(M[0]).tolist() == sorted(kept), tau
        assert abs(m[0] - margin) < 1e-12, (tau, m[0])
    M, m = orc.select_blocks_cdf(S, 0.95, 4, 0, 0)           # everything taken: no cut, no margin
    assert M.all() and m[0] == np.inf


def test_layer_with_cdf_selection_equals_library_masked_attention():
    import torch
    rng = np.random.default_rng(21)
    T, H, W, d, b = 3, 8, 8, 8, 16
    # block means of distinct sizes, so that the rows' score distributions (and lengths) differ
    X = [rng.standard_normal((T * H * W, d)) + (rng.uniform(0, 5, (T * H * W // b, 1, 1)) * rng.standard_normal((T * H * W // b, 1, d))).repeat(b, 1).reshape(-1, d)
         for _ in range(3)]
    r = orc.layer(*X, T=T, H=H, W=W, block=b, sparsity=0.5, sink_frames=1, window=(1, 2, 8), cdf_threshold=0.6)
    assert r["k_row"] == r["M"].shape[0] and len(set(r["M"][:8].sum(1))) > 1      # row lengths vary
    inv = orc.inverse_table(r["perm"])
    allow = torch.from_numpy(r["M"][inv // b][:, inv // b])
    want = torch.nn.functional.scaled_dot_product_attention(*(torch.from_numpy(x)[None] for x in X), attn_mask=allow[None])[0]
    assert np.abs(r["O"] - want.numpy()).max() < 1e-12


def test_rectangular_selection_vs_brute_force():
    """Different block sizes for Q and K: the mask is Tq x Tk with separate sink ranges."""
    rng = np.random.default_rng(31)
    Tq, Tk, k_sel = 7, 13, 4
    S = rng.standard_normal((Tq, Tk))
    rows, cols = (5, 7), (10, 13)
    M = orc.select_blocks(S, k_sel, *rows, sink_k=cols)
    gap = orc.selection_gap(S, k_sel, *rows, sink_k=cols)
    for i in range(Tq):
        if rows[0] <= i < rows[1]:
            assert M[i].all() and gap[i] == np.inf
            continue
        cand = sorted(range(cols[0]), key=lambda j: (-S[i, j], j))
        want = set(cand[:k_sel]) | set(range(*cols))
        assert set(np.flatnonzero(M[i])) == want
        assert abs(gap[i] - (S[i, cand[k_sel - 1]] - S[i, cand[k_sel]])) < 1e-15
    Mc, _ = orc.select_blocks_cdf(S * 5, 0.6, 16, *rows, sink_k=cols)
    assert Mc.shape == (Tq, Tk) and Mc[:, 10:].all() and Mc[5:].all()
    assert np.array_equal(Mc[:5], _cdf_by_loops_rect(S * 5, 0.6, 16, cols)[:5])


def _cdf_by_loops_rect(S, tau, d, cols):
    M = np.zeros(S.shape, dtype=bool)
    for i in range(S.shape[0]):
        cand = list(range(cols[0]))
        w = {j: np.exp(S[i, j] / np.sqrt(d)) for j in cand}
        total, taken, mass = sum(w.values()), [], 0.0
        while cand and (not taken or mass < tau * total):
            best = max(cand, key=lambda j: (S[i, j], -j))
            cand.remove(best); taken.append(best); mass += w[best]
        M[i, taken] = True
        M[i, cols[0]:cols[1]] = True
    return M
