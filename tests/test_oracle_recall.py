"""Diagnostic (CPU, oracle only): how much of the dense attention probability mass the predicted
block mask keeps, with the window permutation of Sec. 3.3 and with plain raster-order blocks.

This is the numeric stand-in for the paper's ablation of the 3-D permutation (its Sec. 4 shows
images, not numbers).  The figures are printed; only properties that must hold are asserted."""
import numpy as np
import pytest

from oracle import rf2_oracle as orc
from paper_2512_24086_amd import inputs
from tests import helpers as hp


def mass_recall(Q, K, r, b):
    """Mean over queries of the dense softmax mass that falls on kept blocks (explicit form in raster
    order, independent of the oracle's own diagnostic, which works on the permuted sequence)."""
    N, d = Q.shape
    inv = orc.inverse_table(r["perm"])
    blk = inv // b
    z = (Q @ K.T) / np.sqrt(d)
    p = np.exp(z - z.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    keep = r["M"][blk][:, blk]
    return float((p * keep).sum(axis=1).mean())


def test_oracle_recall_diagnostic_is_pinned():
    """attention_mass_recall: a mask of ones keeps everything, an empty mask nothing, equal logits give the
    kept share of keys (ragged last block counted by its real keys), and on a real case it equals the
    explicit raster-order computation above; a sample of queries is the mean over exactly those rows."""
    rng = np.random.default_rng(5)
    N, d, b = 150, 8, 32                                   # 5 blocks, the last with 22 rows
    Q, K = rng.standard_normal((N, d)), rng.standard_normal((N, d))
    Tb = orc.n_blocks(N, b)
    assert abs(orc.attention_mass_recall(Q, K, np.ones((Tb, Tb), bool), b) - 1.0) < 1e-12
    assert orc.attention_mass_recall(Q, K, np.zeros((Tb, Tb), bool), b) == 0.0
    M = np.zeros((Tb, Tb), bool); M[:, 1] = True; M[:, 4] = True       # blocks of 32 and 22 keys
    assert abs(orc.attention_mass_recall(np.zeros((N, d)), K, M, b) - (32 + 22) / 150) < 1e-12
    # rectangular blocks: 3 Q blocks of 64 rows over 5 K blocks of 32
    M2 = np.zeros((3, Tb), bool); M2[0, 0] = True; M2[1, :] = True
    want = (64 * 32 / 150 + 64 * 1.0 + 22 * 0.0) / 150
    assert abs(orc.attention_mass_recall(np.zeros((N, d)), K, M2, 64, bk=32) - want) < 1e-12
    wl = inputs.WORKLOADS["tiny"]
    q, k, v = inputs.make_qkv(wl)
    Qh, Kh, Vh = (hp.f64(x[0, 1]) for x in (q, k, v))
    r = orc.layer(Qh, Kh, Vh, T=wl.T, H=wl.H, W=wl.W, block=wl.block, sparsity=0.5, sink_frames=1)
    assert abs(orc.attention_mass_recall(r["Qp"], r["Kp"], r["M"], wl.block) - mass_recall(Qh, Kh, r, wl.block)) < 1e-12
    rows = [3, 77, 700, 1535]
    each = [orc.attention_mass_recall(r["Qp"], r["Kp"], r["M"], wl.block, queries=[n]) for n in rows]
    assert abs(orc.attention_mass_recall(r["Qp"], r["Kp"], r["M"], wl.block, queries=rows) - np.mean(each)) < 1e-12


@pytest.mark.parametrize("name,heads", [("image", (5,)), ("video480p", (11,)), ("video720p", (23,))])
def test_recall_on_the_real_workloads(name, heads):
    """One head of the image / 480p / 720p workloads, 256 seeded query rows: mass kept by the predicted mask
    with the window order of Sec. 3.3 and with raster-order blocks, next to the kept density (the
    recall of a mask that knows nothing).  Printed; asserted only: better than knowing nothing."""
    wl = inputs.WORKLOADS[name]
    rng = np.random.default_rng(wl.index)
    for h in heads:
        Q, K, _ = (hp.f64(x[0, 0]) for x in inputs.make_qkv(wl, heads=[h]))
        N = wl.N
        rows = np.sort(rng.choice(N, 256, replace=False))
        out = {}
        for label, window in (("windows", orc.default_window(wl.block, wl.T > 1)), ("raster", (1, 1, wl.block))):
            perm = orc.perm_table(wl.T, wl.H, wl.W, *window, wl.sink_frames, True)
            Qp, Kp = orc.permute(Q, perm), orc.permute(K, perm)
            S_hat = orc.block_scores(orc.pool_blocks(Qp, wl.block), orc.pool_blocks(Kp, wl.block))
            Tb = orc.n_blocks(N, wl.block)
            sb, se = orc.sink_block_range(N, wl.H * wl.W, wl.block, wl.sink_frames)
            k_row, k_sel = orc.budget(Tb, se - sb, wl.sparsity)
            M = orc.select_blocks(S_hat, k_sel, sb, se)
            out[label] = orc.attention_mass_recall(Qp, Kp, M, wl.block, queries=rows)
            density = M[rows // wl.block].mean()
        print(f"\n[recall] {name} head {h} s={wl.sparsity}: kept density on the sampled rows {density:.3f}; dense "
              f"attention mass kept with window blocks {out['windows']:.4f}, with raster blocks {out['raster']:.4f}")
        assert out["windows"] > density - 0.02 and out["raster"] > density - 0.02


@pytest.mark.parametrize("name,sparsity", [("tiny", 0.5), ("tiny", 0.6)])
def test_recall_with_and_without_window_permutation(name, sparsity):
    wl = inputs.WORKLOADS[name]
    q, k, v = inputs.make_qkv(wl)
    out = {}
    for label, window in (("windows", None), ("raster", (1, 1, wl.block))):
        rec = []
        for h in range(wl.heads):
            Q, K, V = (hp.f64(x[0, h]) for x in (q, k, v))
            r = orc.layer(Q, K, V, T=wl.T, H=wl.H, W=wl.W, block=wl.block, sparsity=sparsity,
                          sink_frames=wl.sink_frames, window=window)
            rec.append(mass_recall(Q, K, r, wl.block))
            assert 0.0 < rec[-1] <= 1.0 + 1e-12
            kept = r["M"].sum() / r["M"].size
        out[label] = float(np.mean(rec))
    print(f"\n[recall] {name} s={sparsity}: kept density {kept:.3f}; attention mass kept with window blocks "
          f"{out['windows']:.4f}, with raster blocks {out['raster']:.4f}")
    dense = orc.layer(Q, K, V, T=wl.T, H=wl.H, W=wl.W, block=wl.block, sparsity=0.0, sink_frames=wl.sink_frames)
    assert abs(mass_recall(Q, K, dense, wl.block) - 1.0) < 1e-12


def test_recall_over_window_shapes_with_local_attention():
    """Window-shape sweep.  With the independent Q and K fields of the workloads the attention rows are
    nearly flat and every block order keeps about the same mass; with Q = K (each token attends to
    tokens whose key resembles its own, i.e. to its smooth-field neighbourhood) the prediction has
    something to find, and the mass kept at equal density depends on the window shape."""
    wl = inputs.WORKLOADS["tiny"]
    _, k, v = inputs.make_qkv(wl)
    shapes = [(4, 4, 4), (2, 4, 8), (2, 2, 16), (1, 8, 8), (1, 4, 16), (1, 1, 64)]      # all of volume b
    table = {}
    for window in shapes:
        rec = []
        for h in range(wl.heads):
            K, V = hp.f64(k[0, h]), hp.f64(v[0, h])
            r = orc.layer(K, K, V, T=wl.T, H=wl.H, W=wl.W, block=wl.block, sparsity=0.5,
                          sink_frames=wl.sink_frames, window=window)
            rec.append(mass_recall(K, K, r, wl.block))
        table[window] = float(np.mean(rec))
        density = r["M"].mean()
        assert density < table[window] <= 1.0 + 1e-12        # better than keeping blocks at random
    print("\n[recall, Q = K] tiny s=0.5, kept density %.3f: " % density
          + ", ".join("%dx%dx%d %.4f" % (*w, table[w]) for w in shapes))
