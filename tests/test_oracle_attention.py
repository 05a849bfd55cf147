"""Pins for the oracle's block-sparse attention and the whole layer (CPU only)."""
import math

import numpy as np
import pytest
import torch

from oracle import rf2_oracle as orc


def sdpa_f64(Q, K, V, allow=None):
    """Library dense / masked softmax attention in fp64 (Sec. 3.1, first paragraph)."""
    q, k, v = (torch.from_numpy(np.ascontiguousarray(x))[None, None] for x in (Q, K, V))
    m = None if allow is None else torch.from_numpy(allow)
    return torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=m)[0, 0].numpy()


def expand_mask(M, N, b):
    return np.kron(M, np.ones((b, b), dtype=bool))[:N, :N]


def loops_masked_softmax(Q, K, V, allow):
    """Per-query masked softmax written out with Python loops."""
    N, d = Q.shape
    O = np.zeros((N, V.shape[1]))
    for r in range(N):
        cols = [c for c in range(N) if allow[r, c]]
        z = [sum(Q[r, e] * K[c, e] for e in range(d)) / math.sqrt(d) for c in cols]
        zmax = max(z)
        w = [math.exp(x - zmax) for x in z]
        tot = sum(w)
        for c, wc in zip(cols, w):
            O[r] += (wc / tot) * V[c]
    return O


def rand_mask(rng, Tb, keep):
    M = rng.random((Tb, Tb)) < keep
    M[np.arange(Tb), rng.integers(0, Tb, Tb)] = True     # at least one block per row
    return M


def test_all_blocks_kept_equals_dense_attention():
    rng = np.random.default_rng(10)
    N, d, b = 333, 32, 64                                  # ragged last block (13 rows)
    Q, K, V = (rng.standard_normal((N, d)) for _ in range(3))
    M = np.ones((orc.n_blocks(N, b),) * 2, dtype=bool)
    O = orc.block_sparse_attention(Q, K, V, M, b)
    assert np.abs(O - sdpa_f64(Q, K, V)).max() < 1e-12


@pytest.mark.parametrize("N,b,keep", [(333, 64, 0.4), (512, 128, 0.5), (200, 64, 0.3)])
def test_masked_equals_library_masked_attention(N, b, keep):
    rng = np.random.default_rng(N)
    d = 16
    Q, K, V = (rng.standard_normal((N, d)) * 2 for _ in range(3))
    M = rand_mask(rng, orc.n_blocks(N, b), keep)
    O, lse = orc.block_sparse_attention(Q, K, V, M, b, return_lse=True)
    allow = expand_mask(M, N, b)
    assert np.abs(O - sdpa_f64(Q, K, V, allow)).max() < 1e-12
    z = np.where(allow, (Q @ K.T) / math.sqrt(d), -np.inf)
    want_lse = np.log(np.exp(z - z.max(1, keepdims=True)).sum(1)) + z.max(1)
    assert np.abs(lse - want_lse).max() < 1e-12


def test_tiny_equals_python_loops():
    rng = np.random.default_rng(11)
    N, d, b = 44, 5, 8                                     # last block has 4 rows
    Q, K, V = (rng.standard_normal((N, d)) for _ in range(3))
    M = rand_mask(rng, orc.n_blocks(N, b), 0.4)
    O = orc.block_sparse_attention(Q, K, V, M, b)
    assert np.abs(O - loops_masked_softmax(Q, K, V, expand_mask(M, N, b))).max() < 1e-12


def test_constant_and_one_hot_values():
    rng = np.random.default_rng(12)
    N, d, b = 320, 8, 64
    Tb = orc.n_blocks(N, b)
    Q, K = rng.standard_normal((N, d)), rng.standard_normal((N, d))
    M = rand_mask(rng, Tb, 0.5)
    assert np.abs(orc.block_sparse_attention(Q, K, np.ones((N, d)), M, b) - 1.0).max() < 1e-13
    V = np.zeros((N, Tb))
    V[np.arange(N), np.arange(N) // b] = 1.0               # value = one-hot(block id)
    O = orc.block_sparse_attention(Q, K, V, M, b)         # -> probability mass per K block
    assert np.abs(O.sum(1) - 1.0).max() < 1e-13
    rows_M = np.repeat(M, b, axis=0)[:N]
    assert (O[~rows_M] == 0).all() and (O[rows_M] > 0).all()


def test_subset_of_q_blocks():
    rng = np.random.default_rng(13)
    N, d, b = 300, 8, 64
    Q, K, V = (rng.standard_normal((N, d)) for _ in range(3))
    M = rand_mask(rng, 5, 0.5)
    full = orc.block_sparse_attention(Q, K, V, M, b)
    part = orc.block_sparse_attention(Q, K, V, M, b, q_blocks=[1, 4])
    assert np.array_equal(part[64:128], full[64:128]) and np.array_equal(part[256:], full[256:])
    assert np.isnan(part[:64]).all() and np.isnan(part[128:256]).all()


def _smooth(rng, T, H, W, d):
    t, h, w = np.meshgrid(np.arange(T) / T, np.arange(H) / H, np.arange(W) / W, indexing="ij")
    X = np.zeros((T * H * W, d))
    for c in range(d):
        f = rng.uniform(-2, 2, 3)
        X[:, c] = np.cos(2 * np.pi * (f[0] * t + f[1] * h + f[2] * w) + rng.uniform(0, 6.28)).ravel()
    return X + 0.3 * rng.standard_normal(X.shape)


def test_layer_sparsity_zero_is_dense_for_any_window_and_sink():
    """With every block kept the layer is plain attention, whatever the permutation."""
    rng = np.random.default_rng(14)
    T, H, W, d, b = 3, 6, 10, 8, 64
    Q, K, V = (_smooth(rng, T, H, W, d) for _ in range(3))
    dense = sdpa_f64(Q, K, V)
    for window, sf, at_end in [((2, 4, 4), 1, True), ((1, 3, 5), 1, False), ((2, 8, 8), 0, True)]:
        r = orc.layer(Q, K, V, T=T, H=H, W=W, block=b, sparsity=0.0, sink_frames=sf,
                      sink_at_end=at_end, window=window)
        assert r["M"].all()
        assert np.abs(r["O"] - dense).max() < 1e-12


def test_layer_sparse_equals_library_attention_in_raster_order():
    """Whole layer vs. library masked attention with the token-level mask built in raster order."""
    rng = np.random.default_rng(15)
    T, H, W, d, b = 4, 8, 8, 8, 32
    N = T * H * W
    Q, K, V = (_smooth(rng, T, H, W, d) for _ in range(3))
    r = orc.layer(Q, K, V, T=T, H=H, W=W, block=b, sparsity=0.5, sink_frames=1, window=(1, 4, 8))
    sb, se = r["sink"]
    assert (sb, se) == (6, 8) and r["M"][:, sb:se].all() and r["M"][sb:se].all()
    assert (r["M"][:sb].sum(1) == r["k_row"]).all()
    inv = orc.inverse_table(r["perm"])
    blk_of = inv // b                                       # block of every raster-order token
    allow = r["M"][blk_of][:, blk_of]
    assert np.abs(r["O"] - sdpa_f64(Q, K, V, allow)).max() < 1e-12
    # first-frame queries see everything; everyone sees the first frame (Sec. 3.4)
    assert allow[:H * W].all() and allow[:, :H * W].all()
    achieved = 1.0 - r["M"].sum() / r["M"].size
    assert achieved >= 0.5


def test_layer_with_text_tokens():
    """Text tokens appended to the video tokens (Sec. 3.4, last paragraph): their rows and columns are
    dense, like the first frame's; the whole layer equals library masked attention over all tokens;
    with every block kept it is plain joint attention."""
    rng = np.random.default_rng(16)
    T, H, W, d, b, text = 4, 8, 8, 8, 32, 21
    Nv, N = T * H * W, T * H * W + text
    Q, K, V = (np.concatenate([_smooth(rng, T, H, W, d), rng.standard_normal((text, d))]) for _ in range(3))
    r = orc.layer(Q, K, V, T=T, H=H, W=W, block=b, sparsity=0.5, sink_frames=1, window=(1, 4, 8), text_tokens=text)
    sb, se = r["sink"]
    assert (sb, se) == (6, 9) and r["M"].shape == (9, 9)      # body 192 tokens = 6 blocks; 64 + 21 dense tokens
    assert r["M"][:, sb:se].all() and r["M"][sb:se].all() and (r["M"][:sb].sum(1) == r["k_row"]).all()
    inv = orc.inverse_table(r["perm"])
    blk_of = inv // b
    allow = r["M"][blk_of][:, blk_of]
    assert np.abs(r["O"] - sdpa_f64(Q, K, V, allow)).max() < 1e-12
    assert allow[Nv:].all() and allow[:, Nv:].all()          # text queries see everything, everyone sees the text
    assert allow[:H * W].all() and allow[:, :H * W].all()    # and the same for the first frame
    dense = orc.layer(Q, K, V, T=T, H=H, W=W, block=b, sparsity=0.0, sink_frames=1, window=(2, 4, 4), text_tokens=text)
    assert dense["M"].all() and np.abs(dense["O"] - sdpa_f64(Q, K, V)).max() < 1e-12
    # text only (an image model with a prompt): the dense range is the text blocks
    im = orc.layer(Q[H * W * 3:], K[H * W * 3:], V[H * W * 3:], T=1, H=H, W=W, block=b, sparsity=0.5,
                   window=(1, 4, 8), text_tokens=text)
    assert im["sink"] == (2, 3) and im["M"][:, 2].all() and im["M"][2].all()


@pytest.mark.parametrize("bq,bk", [(32, 16), (16, 32), (64, 16)])
def test_layer_with_different_q_and_k_blocks(bq, bk):
    """b_q != b_k (Sec. 3.1): the whole layer equals library masked attention whose token-level mask is
    built from the Q block of the query and the K block of the key; sink rows/columns are dense; with
    every block kept it is plain attention."""
    rng = np.random.default_rng(bq * 100 + bk)
    T, H, W, d = 4, 8, 8, 8
    N = T * H * W
    Q, K, V = (_smooth(rng, T, H, W, d) for _ in range(3))
    r = orc.layer(Q, K, V, T=T, H=H, W=W, block=bq, block_k=bk, sparsity=0.5, sink_frames=1, window=(1, 4, 8))
    Tq, Tk = N // bq, N // bk
    assert r["M"].shape == (Tq, Tk) and r["qbar"].shape[0] == Tq and r["kbar"].shape[0] == Tk
    (sb, se), (kb, ke) = r["sink"], r["sink_k"]
    assert (se, ke) == (Tq, Tk) and sb * bq == kb * bk == 3 * H * W       # body = 3 frames, block aligned here
    assert r["M"][sb:].all() and r["M"][:, kb:].all() and (r["M"][:sb].sum(1) == r["k_row"]).all()
    assert 1.0 - r["M"].sum() / r["M"].size >= 0.5
    inv = orc.inverse_table(r["perm"])
    allow = r["M"][inv // bq][:, inv // bk]
    assert np.abs(r["O"] - sdpa_f64(Q, K, V, allow)).max() < 1e-12
    dense = orc.layer(Q, K, V, T=T, H=H, W=W, block=bq, block_k=bk, sparsity=0.0, sink_frames=1, window=(2, 4, 4))
    assert dense["M"].all() and np.abs(dense["O"] - sdpa_f64(Q, K, V)).max() < 1e-12
