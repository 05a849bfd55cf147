"""CPU oracle for the RainFusion2.0 block-sparse attention layer (fp64, NumPy).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
check and the benchmark's CPU-baseline leg may import it.  It shares no code,
table or helper with the HIP library and never imports it.

It is a plain, slow, step-by-step transcription of what one attention layer of
the method computes, in the paper's order:

  token permutation (Sec. 3.3, Sec. 3.4 last paragraph)
  -> block representative tokens            (Sec. 3.2, eqs. 5, 6)
  -> block scores                           (Sec. 3.2, eq. 7)
  -> top-n block selection + first-frame sink (Sec. 3.2, eq. 8; Sec. 3.4)
  -> block-sparse flash attention           (Sec. 3.1, eqs. 1-4 and the skip rule)
  -> inverse permutation                    (implied by Sec. 3.3)

All floating point work is float64 on the exact values of the bf16 inputs.
Every function works on ONE (batch, head) slice: 2-D arrays [N, d].

Pins (see tests/test_oracle_*.py): permutation vs. hand-written fixtures, a
nested-loop window enumeration, bijection and special cases; budget arithmetic
vs. a table of independently derived sizes; selection vs. a repeated-maximum
brute force and hand-built ties; attention vs. a library dense/masked softmax
attention in fp64, explicit per-query Python loops, and closed-form cases
(V == 1, one-hot V).  Fidelity of the window order to the authors' unpublished
permutation: parity unpinned (Sec. 3.3 defers its details).
"""
from __future__ import annotations

import math

import numpy as np

BUDGET_GLOBAL = 0
BUDGET_ROW_INCL_SINK = 1
BUDGET_ROW_PLUS_SINK = 2


# --------------------------------------------------------------------------
# inputs
# --------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 numbers given as their 16-bit patterns."""
    u = np.asarray(bits).view(np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# Sec. 3.3 / Sec. 3.4: spatiotemporal window permutation, sink relocated
# --------------------------------------------------------------------------
def default_window(block: int, video: bool) -> tuple[int, int, int]:
    """Window whose volume equals the block size, so one interior window is one
    block (the paper gives no shape; this is a parameter of the method)."""
    table = {(256, True): (4, 8, 8), (256, False): (1, 16, 16),
             (128, True): (2, 8, 8), (128, False): (1, 8, 16),
             (64, True): (4, 4, 4), (64, False): (1, 8, 8)}
    return table[(block, video)]


def _window_order(frames: np.ndarray, H: int, W: int, wt: int, wh: int, ww: int) -> np.ndarray:
    """Source indices of the tokens of `frames` (consecutive frame numbers)
    listed window by window (windows in raster order over the window grid) and
    in raster order inside each window.  Edge windows are simply smaller."""
    t0 = int(frames[0])
    t, h, w = np.meshgrid(frames, np.arange(H), np.arange(W), indexing="ij")
    t, h, w = t.ravel(), h.ravel(), w.ravel()
    tp = t - t0
    # np.lexsort sorts by the LAST key first.
    order = np.lexsort((w % ww, h % wh, tp % wt, w // ww, h // wh, tp // wt))
    return ((t * H + h) * W + w)[order]


def perm_table(T: int, H: int, W: int, wt: int, wh: int, ww: int,
               sink_frames: int = 0, sink_at_end: bool = True, text_tokens: int = 0) -> np.ndarray:
    """perm[p] = input index of the token placed at permuted position p.  The
    input lists the video tokens in raster order n=(t*H+h)*W+w, then
    `text_tokens` tokens of the other modality.  Body frames (t >= sink_frames)
    use 3-D windows (wt,wh,ww); sink frames use 2-D windows (1,wh,ww) frame by
    frame and are placed after the body (Sec. 3.4, last paragraph) or before it
    (Fig. 1).  Text tokens keep their order and come last, next to the sink
    frame (Sec. 3.4, last paragraph: both take part in full attention)."""
    _check_tail(sink_frames, sink_at_end, text_tokens)
    body = _window_order(np.arange(sink_frames, T), H, W, wt, wh, ww)
    parts = [body]
    if sink_frames > 0:
        sink = _window_order(np.arange(0, sink_frames), H, W, 1, wh, ww)
        parts = [body, sink] if sink_at_end else [sink, body]
    parts.append(T * H * W + np.arange(text_tokens))
    return np.concatenate(parts).astype(np.int64)


def _check_tail(sink_frames: int, sink_at_end: bool, text_tokens: int) -> None:
    """The always-dense tokens (sink frames, text) must form ONE run of the
    permuted sequence; a sink at the front plus text at the end would be two."""
    if text_tokens < 0:
        raise ValueError("text_tokens must be >= 0")
    if text_tokens > 0 and sink_frames > 0 and not sink_at_end:
        raise ValueError("text tokens need the sink frames at the end of the sequence")


def inverse_table(perm: np.ndarray) -> np.ndarray:
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size, dtype=perm.dtype)
    return inv


def permute(X: np.ndarray, perm: np.ndarray) -> np.ndarray:
    """X_p[p] = X[perm[p]]."""
    return X[perm]


def unpermute(Xp: np.ndarray, perm: np.ndarray) -> np.ndarray:
    """X[perm[p]] = X_p[p]."""
    X = np.empty_like(Xp)
    X[perm] = Xp
    return X


# --------------------------------------------------------------------------
# blocks, sink block range, budget
# --------------------------------------------------------------------------
def n_blocks(N: int, b: int) -> int:
    return -(-N // b)


def block_slice(i: int, N: int, b: int) -> slice:
    return slice(i * b, min((i + 1) * b, N))


def sink_block_range(N: int, frame_tokens: int, b: int, sink_frames: int,
                     sink_at_end: bool = True, text_tokens: int = 0) -> tuple[int, int]:
    """[begin, end) of the blocks that hold at least one always-dense token: a
    sink-frame token or a text token (N counts the text tokens too)."""
    _check_tail(sink_frames, sink_at_end, text_tokens)
    n_sink = sink_frames * frame_tokens
    Tb = n_blocks(N, b)
    if n_sink + text_tokens == 0:
        return (0, 0)
    if sink_at_end or n_sink == 0:
        return ((N - n_sink - text_tokens) // b, Tb)
    return (0, -(-n_sink // b))


def budget(Tb: int, n_sink_blocks: int, sparsity: float, mode: int = BUDGET_GLOBAL,
           Tk: int | None = None, n_sink_k: int | None = None) -> tuple[int, int]:
    """(k_row, k_sel): K blocks kept per non-sink row in total, and those chosen
    by score among the non-sink columns.  `sparsity` is taken as a float32
    value; the arithmetic is IEEE double.  The mask has Tb rows (Q blocks, of
    which n_sink_blocks are sink rows) and Tk columns (K blocks, n_sink_k sink
    columns); by default it is square (Sec. 3.1 allows b_q != b_k).

    GLOBAL: the target is the skipped fraction of the whole Tb x Tk mask, sink
    rows and columns included.  ROW_INCL_SINK: each row keeps ceil((1-s)Tk)
    blocks, the sink among them.  ROW_PLUS_SINK: each row selects ceil((1-s)Tk)
    blocks on top of the sink."""
    Tk = Tb if Tk is None else Tk
    nSk = n_sink_blocks if n_sink_k is None else n_sink_k
    keep = 1.0 - float(np.float32(sparsity))
    nS = n_sink_blocks
    if nS >= Tb:
        return (Tk, 0)
    if mode == BUDGET_GLOBAL:
        k_row = int(math.floor((keep * Tb * Tk - float(nS) * Tk) / float(Tb - nS)))
    elif mode == BUDGET_ROW_INCL_SINK:
        k_row = int(math.ceil(keep * Tk))
    elif mode == BUDGET_ROW_PLUS_SINK:
        k_row = int(math.ceil(keep * Tk)) + nSk
    else:
        raise ValueError("budget mode")
    k_row = min(max(k_row, nSk, 1), Tk)
    return (k_row, k_row - nSk)


def kept_pairs(Tb: int, n_sink_blocks: int, k_row: int, Tk: int | None = None) -> int:
    return (Tb - n_sink_blocks) * k_row + n_sink_blocks * (Tb if Tk is None else Tk)


# --------------------------------------------------------------------------
# Sec. 3.2: representative tokens, block scores, top-n selection; Sec. 3.4 sink
# --------------------------------------------------------------------------
def pool_blocks(Xp: np.ndarray, b: int) -> np.ndarray:
    """Eqs. (5), (6): mean over the rows of each block (a ragged last block is
    averaged over the rows it really has)."""
    N = Xp.shape[0]
    return np.stack([Xp[block_slice(i, N, b)].mean(axis=0) for i in range(n_blocks(N, b))])


def block_scores(qbar: np.ndarray, kbar: np.ndarray) -> np.ndarray:
    """Eq. (7): S_hat[i, j] = <qbar_i, kbar_j>, no scaling."""
    return qbar @ kbar.T


def select_blocks(S_hat: np.ndarray, k_sel: int, sink_begin: int, sink_end: int, sink_k=None) -> np.ndarray:
    """Eq. (8) with the sink of Sec. 3.4.  Non-sink row i keeps the k_sel
    non-sink columns with the largest S_hat[i, :] (equal scores: lower column
    first) and every sink column; sink rows keep every column.  Rows are Q
    blocks with sink range [sink_begin, sink_end); columns are K blocks with
    sink range sink_k (the same range unless b_q != b_k)."""
    Tq, Tk = S_hat.shape
    kb, ke = (sink_begin, sink_end) if sink_k is None else sink_k
    M = np.zeros((Tq, Tk), dtype=bool)
    cand = np.array([j for j in range(Tk) if not (kb <= j < ke)], dtype=np.int64)
    for i in range(Tq):
        if sink_begin <= i < sink_end:
            M[i, :] = True
            continue
        s = S_hat[i, cand]
        order = np.lexsort((cand, -s))          # by -score, then by column
        M[i, cand[order[:k_sel]]] = True
        M[i, kb:ke] = True
    return M


def selection_gap(S_hat: np.ndarray, k_sel: int, sink_begin: int, sink_end: int, sink_k=None) -> np.ndarray:
    """Per row: (k_sel-th largest candidate score) - ((k_sel+1)-th largest);
    +inf where the row has no boundary (sink row, or every candidate kept)."""
    Tq, Tk = S_hat.shape
    kb, ke = (sink_begin, sink_end) if sink_k is None else sink_k
    cand = np.array([j for j in range(Tk) if not (kb <= j < ke)], dtype=np.int64)
    gap = np.full(Tq, np.inf)
    if k_sel <= 0 or k_sel >= cand.size:
        return gap
    for i in range(Tq):
        if sink_begin <= i < sink_end:
            continue
        s = np.sort(S_hat[i, cand])[::-1]
        gap[i] = s[k_sel - 1] - s[k_sel]
    return gap


def select_blocks_cdf(S_hat: np.ndarray, tau: float, d: int, sink_begin: int, sink_end: int, sink_k=None):
    """Threshold variant of the selection (the cumulative-mass rule Sec. 2 describes for
    online adaptive patterns, applied to the block scores of eq. 7): for every non-sink
    row, softmax over the non-sink columns of S_hat / sqrt(d); the columns are taken in
    the order of eq. (8) (largest score first, equal scores: lower column first) until
    their cumulative probability reaches tau; at least one is taken.  Sink columns are
    always kept, sink rows keep every column (Sec. 3.4).  Returns (M, margin): margin[i]
    = distance between tau and the nearer of the cumulative probabilities just before and
    just after the last column taken (+inf for sink rows and rows that take everything) --
    a row whose margin is tiny may legitimately be cut one column earlier or later by
    arithmetic of lower precision."""
    if not (0.0 < tau < 1.0):
        raise ValueError("tau must lie strictly between 0 and 1")
    Tq, Tk = S_hat.shape
    kb, ke = (sink_begin, sink_end) if sink_k is None else sink_k
    M = np.zeros((Tq, Tk), dtype=bool)
    margin = np.full(Tq, np.inf)
    cand = np.array([j for j in range(Tk) if not (kb <= j < ke)], dtype=np.int64)
    for i in range(Tq):
        if sink_begin <= i < sink_end or cand.size == 0:
            M[i, :] = True
            continue
        z = S_hat[i, cand] / math.sqrt(d)
        p = np.exp(z - z.max())
        p /= p.sum()
        order = np.lexsort((cand, -z))
        cum = np.cumsum(p[order])
        n = int(np.argmax(cum >= tau)) + 1 if (cum >= tau).any() else cand.size
        M[i, cand[order[:n]]] = True
        M[i, kb:ke] = True
        if n < cand.size:
            before = cum[n - 2] if n >= 2 else 0.0
            margin[i] = min(abs(cum[n - 1] - tau), abs(tau - before))
    return M, margin


def mask_to_lists(M: np.ndarray) -> list[np.ndarray]:
    """Ascending kept-column list of every row."""
    return [np.flatnonzero(M[i]).astype(np.int32) for i in range(M.shape[0])]


# --------------------------------------------------------------------------
# Sec. 3.1: block-sparse flash attention, eqs. (1)-(4) + skip rule
# --------------------------------------------------------------------------
def block_sparse_attention(Qp: np.ndarray, Kp: np.ndarray, Vp: np.ndarray, M: np.ndarray,
                           b: int, q_blocks=None, return_lse: bool = False, bk: int | None = None):
    """Output rows of the requested Q blocks (default: all), by the online
    recurrences (Q blocks of b rows, K/V blocks of bk rows, bk = b unless
    given; M is [ceil(N/b), ceil(N/bk)]): for each kept block j in ascending order
        S = Q_i K_j^T / sqrt(d)                                   (1)
        m_new = max(m, rowmax S),  P = exp(S - m_new)             (2)
        l = exp(m - m_new) l + rowsum P                           (3)
        O = diag(exp(m - m_new)) O + P V_j                        (4)
    and finally O_i = diag(l)^-1 O.  Blocks with M[i, j] == 0 are skipped."""
    N, d = Qp.shape
    bk = b if bk is None else bk
    Tb, Tk = n_blocks(N, b), n_blocks(N, bk)
    assert M.shape == (Tb, Tk)
    rows = range(Tb) if q_blocks is None else q_blocks
    dv = Vp.shape[1]
    O = np.zeros((N, dv))
    lse = np.full(N, np.nan)
    inv_sqrt_d = 1.0 / math.sqrt(d)
    for i in rows:
        qs = block_slice(i, N, b)
        Qi = Qp[qs]
        m = np.full((Qi.shape[0], 1), -np.inf)
        l = np.zeros((Qi.shape[0], 1))
        acc = np.zeros((Qi.shape[0], dv))
        for j in range(Tk):
            if not M[i, j]:
                continue
            ks = block_slice(j, N, bk)
            S = (Qi @ Kp[ks].T) * inv_sqrt_d
            m_new = np.maximum(m, S.max(axis=1, keepdims=True))
            P = np.exp(S - m_new)
            scale = np.exp(m - m_new)
            l = scale * l + P.sum(axis=1, keepdims=True)
            acc = scale * acc + P @ Vp[ks]
            m = m_new
        O[qs] = acc / l
        lse[qs] = (m + np.log(l))[:, 0]
    if q_blocks is not None:
        keep = np.zeros(N, dtype=bool)
        for i in q_blocks:
            keep[block_slice(i, N, b)] = True
        O[~keep] = np.nan
    return (O, lse) if return_lse else O


# --------------------------------------------------------------------------
# diagnostic: how much of the dense attention the block mask keeps
# --------------------------------------------------------------------------
def attention_mass_recall(Qp: np.ndarray, Kp: np.ndarray, M: np.ndarray, b: int, bk: int | None = None,
                          queries=None) -> float:
    """Mean, over the query rows `queries` of the permuted sequence (default: all), of the
    probability mass that DENSE attention (softmax(q K^T / sqrt(d)) over every key, Sec. 3.1
    first paragraph) puts on the keys of the K blocks the mask keeps for that query's Q block.
    1 for a mask of ones; the kept share of keys when all logits are equal."""
    N, d = Qp.shape
    bk = b if bk is None else bk
    rows = np.arange(N) if queries is None else np.asarray(queries)
    z = (Qp[rows] @ Kp.T) / math.sqrt(d)
    p = np.exp(z - z.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    kept = M[rows // b][:, np.arange(N) // bk]            # [queries, keys]: is the key's block kept for this query
    return float((p * kept).sum(axis=1).mean())


# --------------------------------------------------------------------------
# whole layer for one head
# --------------------------------------------------------------------------
def layer(Q: np.ndarray, K: np.ndarray, V: np.ndarray, *, T: int, H: int, W: int, block: int,
          sparsity: float, sink_frames: int = 0, sink_at_end: bool = True,
          window=None, budget_mode: int = BUDGET_GLOBAL, q_blocks=None, text_tokens: int = 0,
          cdf_threshold: float | None = None, block_k: int | None = None) -> dict:
    """All stages for one (batch, head).  Q, K, V: [N, d] float64, the video
    tokens in [T,H,W] raster order followed by `text_tokens` text tokens.
    Returns every intermediate."""
    N = T * H * W + text_tokens
    assert Q.shape[0] == N
    wt, wh, ww = window if window is not None else default_window(block, T > 1)
    perm = perm_table(T, H, W, wt, wh, ww, sink_frames, sink_at_end, text_tokens)
    Qp, Kp, Vp = permute(Q, perm), permute(K, perm), permute(V, perm)
    bk = block if block_k is None else block_k            # Q blocks of `block` rows, K/V blocks of bk rows
    qbar, kbar = pool_blocks(Qp, block), pool_blocks(Kp, bk)
    S_hat = block_scores(qbar, kbar)
    Tb, Tk = n_blocks(N, block), n_blocks(N, bk)
    sb, se = sink_block_range(N, H * W, block, sink_frames, sink_at_end, text_tokens)
    sink_k = sink_block_range(N, H * W, bk, sink_frames, sink_at_end, text_tokens)
    k_row, k_sel = budget(Tb, se - sb, sparsity, budget_mode, Tk, sink_k[1] - sink_k[0])
    if cdf_threshold is None:
        M = select_blocks(S_hat, k_sel, sb, se, sink_k)
        gap = selection_gap(S_hat, k_sel, sb, se, sink_k)
    else:                       # cumulative-mass selection: row lengths vary, the budget does not apply
        M, gap = select_blocks_cdf(S_hat, cdf_threshold, Q.shape[1], sb, se, sink_k)
        k_row, k_sel = Tk, 0
    Op, lse = block_sparse_attention(Qp, Kp, Vp, M, block, q_blocks=q_blocks, return_lse=True, bk=bk)
    O = unpermute(Op, perm)
    return dict(perm=perm, Qp=Qp, Kp=Kp, Vp=Vp, qbar=qbar, kbar=kbar, S_hat=S_hat, M=M,
                sink=(sb, se), sink_k=sink_k, k_row=k_row, k_sel=k_sel, Op=Op, lse=lse, O=O,
                gap=gap)
