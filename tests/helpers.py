"""Shared helpers of the GPU parity tests (no test cases here)."""
import numpy as np
import torch

from oracle import rf2_oracle as orc
from paper_2512_24086_amd import inputs, rf2

# Tolerances of the attention output vs. the fp64 oracle (bf16 operands, fp32 accumulation,
# probabilities and outputs rounded to bf16: |O| <= max|V| ~ 4, bf16 half-ulp at 4 is 2^-7 = 7.8e-3).
ATTN_MAX_ABS = 2e-2
ATTN_MEAN_ABS = 2e-3
TIE_GAP = 1e-3          # rows whose selection-boundary score gap is below this may differ
CDF_TIE = 2e-5          # cumulative-mass selection: rows cut within this (normalised mass) of tau may differ (fp32 sums of <= 2048 terms)


def f64(t: torch.Tensor) -> np.ndarray:
    """Exact fp64 values of a bf16 tensor (through its bit pattern)."""
    return orc.bf16_bits_to_f64(inputs.bf16_bits(t)).reshape(tuple(t.shape))


def rho(r):
    return (r & 3) | ((r & 4) << 1) | ((r & 8) >> 1)


def kp_to_rows(kp: np.ndarray) -> np.ndarray:
    """Decode the K operand tiles [Tb, b/64, d/8, 64, 8] of one head into row-major [Tb*b, d]."""
    Tb, parts, C, _, _ = kp.shape
    b, KH = parts * 64, parts * 32
    r = np.arange(b)
    part, slot = (r % KH) // 32, (r // KH) * 32 + r % 32
    rows = kp[:, part, :, slot, :]                     # [b, Tb, C, 8]
    return np.transpose(rows, (1, 0, 2, 3)).reshape(Tb * b, C * 8)


def vp_to_rows(vp: np.ndarray) -> np.ndarray:
    """Decode the V operand tiles [Tb, b/64, 8, d, 8] of one head into row-major [Tb*b, d]."""
    Tb, parts, _, d, _ = vp.shape
    b, KH = parts * 64, parts * 32
    s = np.arange(b)                                  # storage position inside the block
    key_of_pos = (s & ~15) + rho(s & 15)
    part, g, e = (s % KH) // 32, (s // KH) * 4 + (s % 32) // 8, s % 8
    by_pos = vp[:, part, g, :, e]                      # [b, Tb, d]
    out = np.empty((Tb, b, d), dtype=vp.dtype)
    out[:, key_of_pos, :] = np.transpose(by_pos, (1, 0, 2))
    return out.reshape(Tb * b, d)


def lists_to_device(M_heads, k_row, Tb, device):
    """Oracle masks [heads][Tq,Tk] -> (blk_idx [1,heads,Tq,k_row], blk_cnt [1,heads,Tq]) tensors."""
    Hh = len(M_heads)
    Tb, Tk = M_heads[0].shape
    idx = np.zeros((1, Hh, Tb, k_row), dtype=np.int32)
    cnt = np.zeros((1, Hh, Tb), dtype=np.int32)
    for h, M in enumerate(M_heads):
        for i in range(Tb):
            cols = np.flatnonzero(M[i]).astype(np.int32)
            if cols.size == Tk:
                cnt[0, h, i] = Tk
                idx[0, h, i, :] = np.arange(k_row)
            else:
                assert cols.size <= k_row
                cnt[0, h, i] = cols.size
                idx[0, h, i, :cols.size] = cols
    return torch.from_numpy(idx).to(device), torch.from_numpy(cnt).to(device)


def gpu_lists_to_mask(blk_idx, blk_cnt, Tb, Tk=None):
    """Device lists of one head -> boolean [Tb,Tk] (Tk = Tb unless given); checks the list format on the way."""
    idx, cnt = blk_idx.cpu().numpy(), blk_cnt.cpu().numpy()
    Tk = Tb if Tk is None else Tk
    M = np.zeros((Tb, Tk), dtype=bool)
    for i in range(Tb):
        if cnt[i] == Tk:
            M[i] = True
        else:
            cols = idx[i, :cnt[i]]
            assert (np.diff(cols) > 0).all(), "block list must be strictly ascending"
            assert cols.min() >= 0 and cols.max() < Tk
            M[i, cols] = True
    return M


def check_exempt_rows(M_gpu, M_ref, S_hat, exempt, sink_cols, *, k_sel=None, d=None):
    """Validity of the rows that are exempt from bit-exactness (several results are correct there,
    but not every result).  Returns how many exempt rows differ from the oracle's.

    Top-n rows (k_sel given; eq. 8): the row keeps exactly k_sel candidates, and every column on
    which the two masks differ has an oracle score within TIE_GAP of the row's k_sel-th largest.
    Cumulative-mass rows (d given): the row is cut at most one column earlier or later than the
    oracle's, and what it keeps is a prefix of the oracle's descending order (columns whose
    oracle scores lie within TIE_GAP of the score at the cut may trade places)."""
    cand = np.flatnonzero(~sink_cols)
    differing = 0
    for i in np.flatnonzero(exempt):
        assert M_gpu[i, sink_cols].all(), (i, "sink columns are always kept")
        s = S_hat[i, cand]
        got, want = M_gpu[i, cand], M_ref[i, cand]
        differing += int(not np.array_equal(got, want))
        if k_sel is not None:
            assert got.sum() == k_sel, (i, got.sum())
            boundary = np.sort(s)[::-1][k_sel - 1]
            off = np.abs(s[got ^ want] - boundary)
            assert (off <= TIE_GAP).all(), (i, off.max())
        else:
            n_got, n_want = int(got.sum()), int(want.sum())
            assert n_got >= 1 and abs(n_got - n_want) <= 1, (i, n_got, n_want)
            order = np.lexsort((cand, -s))
            prefix = np.zeros_like(got)
            prefix[order[:n_got]] = True
            off = np.abs(s[got ^ prefix] - s[order[n_got - 1]])
            assert (off <= TIE_GAP).all(), (i, off.max())
    return differing


def make_plan(wl: inputs.Workload, sparsity=None, **kw):
    args = dict(batch=wl.batch, heads=wl.heads, head_dim=wl.head_dim, T=wl.T, H=wl.H, W=wl.W, block=wl.block,
                sparsity=wl.sparsity if sparsity is None else sparsity, sink_frames=wl.sink_frames,
                text_tokens=wl.text_tokens)
    args.update(kw)
    return rf2.Plan(**args)


def oracle_layer(wl, q, k, v, head, plan, q_blocks=None, sparsity=None):
    c = plan.cfg
    Q, K, V = (f64(x[0, head]) for x in (q, k, v))
    return orc.layer(Q, K, V, T=c.T, H=c.H, W=c.W, block=c.block, sparsity=c.sparsity, sink_frames=c.sink_frames,
                     sink_at_end=bool(c.sink_at_end), window=(plan.info.wt, plan.info.wh, plan.info.ww),
                     budget_mode=c.budget_mode, q_blocks=q_blocks, text_tokens=c.text_tokens,
                     cdf_threshold=float(c.cdf_threshold) if c.select_mode == rf2.RF2_SELECT_CDF else None,
                     block_k=plan.info.block_k)
