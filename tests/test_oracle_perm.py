"""Pins for the oracle's permutation, block and budget arithmetic (CPU only)."""
import os

import numpy as np
import pytest

from oracle import rf2_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield [f.strip() for f in line.split("|")]


@pytest.mark.parametrize("row", list(_rows("perm_examples.txt")), ids=lambda r: r[0])
def test_perm_matches_hand_written_examples(row):
    _, thw, win, sink, perm = row[:5]
    text = int(row[5]) if len(row) > 5 else 0
    T, H, W = map(int, thw.split())
    wt, wh, ww = map(int, win.split())
    sf, at_end = map(int, sink.split())
    want = np.array(list(map(int, perm.split())))
    got = orc.perm_table(T, H, W, wt, wh, ww, sf, bool(at_end), text)
    assert got.tolist() == want.tolist()


def brute_force_perm(T, H, W, wt, wh, ww, sink_frames, sink_at_end):
    """Independent enumeration: nested loops over windows then over the tokens in a window."""
    def frames_order(t_lo, t_hi, wt_):
        out = []
        for a in range(t_lo, t_hi, wt_):
            for b in range(0, H, wh):
                for c in range(0, W, ww):
                    for t in range(a, min(a + wt_, t_hi)):
                        for h in range(b, min(b + wh, H)):
                            for w in range(c, min(c + ww, W)):
                                out.append((t * H + h) * W + w)
        return out
    body = frames_order(sink_frames, T, wt)
    sink = frames_order(0, sink_frames, 1)
    return body + sink if sink_at_end else sink + body


def closed_form_pos(T, H, W, wt, wh, ww, sink_frames, sink_at_end, t, h, w):
    """Position of token (t,h,w) from the closed form with truncated edge windows."""
    def pos_in(Tn, tp, wt_):
        a, b, c = tp // wt_, h // wh, w // ww
        u, v, x = tp % wt_, h % wh, w % ww
        et, eh, ew = min(wt_, Tn - a * wt_), min(wh, H - b * wh), min(ww, W - c * ww)
        return a * wt_ * H * W + et * (b * wh * W) + et * eh * (c * ww) + u * eh * ew + v * ew + x
    Tb = T - sink_frames
    if t >= sink_frames:
        p = pos_in(Tb, t - sink_frames, wt)
        return p if sink_at_end else p + sink_frames * H * W
    p = pos_in(sink_frames, t, 1)
    return p + Tb * H * W if sink_at_end else p


CASES = [
    (5, 7, 9, 2, 4, 4, 0, True), (5, 7, 9, 2, 4, 4, 1, True), (5, 7, 9, 2, 4, 4, 1, False),
    (6, 16, 16, 4, 4, 4, 1, True), (1, 10, 13, 1, 8, 16, 0, True), (4, 5, 3, 3, 2, 2, 2, True),
    (3, 8, 8, 2, 8, 8, 1, True), (7, 3, 5, 2, 2, 3, 1, False),
]


@pytest.mark.parametrize("case", CASES)
def test_perm_vs_brute_force_and_closed_form(case):
    T, H, W, wt, wh, ww, sf, at_end = case
    perm = orc.perm_table(*case)
    assert perm.tolist() == brute_force_perm(*case)
    assert sorted(perm.tolist()) == list(range(T * H * W))          # bijection
    inv = orc.inverse_table(perm)
    for t in range(T):
        for h in range(H):
            for w in range(W):
                assert inv[(t * H + h) * W + w] == closed_form_pos(*case, t, h, w)


def test_identity_windows_and_rotation():
    T, H, W = 4, 6, 5
    # a window covering the whole body, or single rows, leaves raster order unchanged
    assert orc.perm_table(T, H, W, T, H, W).tolist() == list(range(T * H * W))
    assert orc.perm_table(T, H, W, 1, 1, W).tolist() == list(range(T * H * W))
    # identity window + sink at end = rotation by one frame
    p = orc.perm_table(T, H, W, 1, 1, W, 1, True)
    assert p.tolist() == list(range(H * W, T * H * W)) + list(range(H * W))


def test_interior_window_is_one_block():
    T, H, W, b = 5, 16, 16, 128
    wt, wh, ww = orc.default_window(b, True)
    assert wt * wh * ww == b
    perm = orc.perm_table(T, H, W, wt, wh, ww, 1, True)
    blk = perm[:b]                       # first window of the body (frames 1,2)
    t, h, w = blk // (H * W), (blk // W) % H, blk % W
    assert set(t) == {1, 2} and h.max() - h.min() == wh - 1 and w.max() - w.min() == ww - 1
    for blk_sz, vid in [(256, True), (256, False), (128, True), (128, False), (64, True), (64, False)]:
        win = orc.default_window(blk_sz, vid)
        assert np.prod(win) == blk_sz and (vid or win[0] == 1)
        # the first interior window fills exactly the first block: a box of the window's shape
        Tg, Hg, Wg = (2 * win[0] if vid else 1), 2 * win[1], 2 * win[2]
        first = orc.perm_table(Tg, Hg, Wg, *win)[:blk_sz]
        t, h, w = first // (Hg * Wg), (first // Wg) % Hg, first % Wg
        assert (t.max() + 1, h.max() + 1, w.max() + 1) == win and len(set(first.tolist())) == blk_sz


def test_round_trip_is_identity():
    rng = np.random.default_rng(0)
    perm = orc.perm_table(5, 7, 9, 2, 4, 4, 1, True)
    X = rng.standard_normal((perm.size, 3))
    assert np.array_equal(orc.unpermute(orc.permute(X, perm), perm), X)
    assert np.array_equal(orc.permute(X, perm)[7], X[perm[7]])
    assert np.array_equal(orc.permute(orc.unpermute(X, perm), perm), X)


@pytest.mark.parametrize("row", list(_rows("config_sizes.txt")), ids=lambda r: r[0])
def test_sizes_of_the_workloads(row):
    _, thw, b, sf, s, N, Tb, sb, nS, k_row, k_sel, kept = row[:12]
    text = int(row[12]) if len(row) > 12 else 0
    T, H, W = map(int, thw.split())
    b, sf = int(b), int(sf)
    assert T * H * W + text == int(N)
    assert orc.n_blocks(int(N), b) == int(Tb)
    begin, end = orc.sink_block_range(int(N), H * W, b, sf, True, text)
    assert end - begin == int(nS)
    if int(nS):
        assert begin == int(sb) and end == int(Tb)
    kr, ks = orc.budget(int(Tb), int(nS), float(s))
    assert (kr, ks) == (int(k_row), int(k_sel))
    assert orc.kept_pairs(int(Tb), int(nS), kr) == int(kept)
    assert 1.0 - int(kept) / int(Tb) ** 2 >= float(s) - 1e-9     # achieved sparsity meets the target


def test_budget_modes_and_extremes():
    assert orc.budget(591, 29, 0.8, orc.BUDGET_ROW_INCL_SINK) == (119, 90)
    assert orc.budget(591, 29, 0.8, orc.BUDGET_ROW_PLUS_SINK) == (148, 119)
    assert orc.budget(32, 0, 0.0) == (32, 32)                   # sparsity 0 keeps everything
    assert orc.budget(24, 4, 0.0) == (24, 20)
    assert orc.budget(32, 0, 0.999) == (1, 1)                   # never below one block
    assert orc.budget(24, 4, 0.99) == (4, 0)                    # never below the sink


def test_sink_block_range_front_and_straddle():
    # 720p: body 72000 tokens -> block 562 holds both body and sink tokens
    assert orc.sink_block_range(75600, 3600, 128, 1, True) == (562, 591)
    assert orc.sink_block_range(75600, 3600, 128, 1, False) == (0, 29)
    assert orc.sink_block_range(4096, 4096, 128, 0, True) == (0, 0)
    perm = orc.perm_table(6, 16, 16, 4, 4, 4, 1, True)
    sb, se = orc.sink_block_range(1536, 256, 64, 1, True)
    first_frame_pos = np.flatnonzero(perm < 256)
    assert set(first_frame_pos // 64) == set(range(sb, se))


def test_text_tokens_stay_in_order_at_the_end_and_are_dense():
    T, H, W, text = 5, 7, 9, 11
    video = orc.perm_table(T, H, W, 2, 4, 4, 1, True)
    both = orc.perm_table(T, H, W, 2, 4, 4, 1, True, text)
    assert both[:T * H * W].tolist() == video.tolist()            # the video part is untouched
    assert both[T * H * W:].tolist() == list(range(T * H * W, T * H * W + text))
    assert sorted(both.tolist()) == list(range(T * H * W + text))
    # every block with a first-frame or text token is in the dense range, and no other block is
    N, b = T * H * W + text, 16
    sb, se = orc.sink_block_range(N, H * W, b, 1, True, text)
    dense_pos = np.flatnonzero((both < H * W) | (both >= T * H * W))
    assert set(dense_pos // b) == set(range(sb, se)) and se == orc.n_blocks(N, b)
    # text without any sink frame: the dense range is the text blocks
    assert orc.sink_block_range(4096 + 77, 4096, 128, 0, True, 77) == (32, 33)
    assert orc.sink_block_range(4096 + 77, 4096, 128, 0, False, 77) == (32, 33)
    with pytest.raises(ValueError):
        orc.perm_table(T, H, W, 2, 4, 4, 1, False, text)          # two separate dense runs: not defined
    with pytest.raises(ValueError):
        orc.sink_block_range(N, H * W, b, 1, False, text)


def test_bf16_decoding():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3DCD, 0x0000, 0x7F80], dtype=np.uint16)
    got = orc.bf16_bits_to_f64(bits)
    assert got[:3].tolist() == [1.0, -1.0, 2.0]
    assert got[3] == 0.10009765625 and got[4] == 0.0 and np.isinf(got[5])


@pytest.mark.parametrize("row", list(_rows("config_sizes_rect.txt")), ids=lambda r: r[0])
def test_sizes_with_different_q_and_k_blocks(row):
    _, thw, bqk, sf, s, N, tqk, sq, sk, kk, kept = row
    T, H, W = map(int, thw.split())
    bq, bk = map(int, bqk.split())
    Tq, Tk = map(int, tqk.split())
    (sbq, nSq), (sbk, nSk) = map(int, sq.split()), map(int, sk.split())
    k_row, k_sel = map(int, kk.split())
    N = int(N)
    assert T * H * W == N and (orc.n_blocks(N, bq), orc.n_blocks(N, bk)) == (Tq, Tk)
    assert orc.sink_block_range(N, H * W, bq, int(sf), True) == (sbq, sbq + nSq) == (sbq, Tq)
    assert orc.sink_block_range(N, H * W, bk, int(sf), True) == (sbk, sbk + nSk) == (sbk, Tk)
    assert orc.budget(Tq, nSq, float(s), orc.BUDGET_GLOBAL, Tk, nSk) == (k_row, k_sel)
    assert orc.kept_pairs(Tq, nSq, k_row, Tk) == int(kept)
    assert 1.0 - int(kept) / (Tq * Tk) >= float(s) - 1e-9
