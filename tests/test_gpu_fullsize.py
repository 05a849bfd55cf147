"""GPU parity at the full workload sizes, in the launch configuration bench.py times.

The oracle cannot run whole 75K-token layers in seconds, so it checks: permutation and
pooling of sampled heads in full, the block mask of sampled heads in full, attention on
sampled Q blocks (first, last/ragged, a sink row, the block straddling body and sink, a few
seeded random ones) with every one of their rows, plus properties that hold at any size.
"""
import numpy as np
import pytest
import torch

from oracle import rf2_oracle as orc
from paper_2512_24086_amd import inputs, rf2
from tests import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda"

CASES = {
    # name: (workload, sparsity, sampled heads)
    "video720p": ("video720p", 0.8, (0, 17, 39)),
    "video480p": ("video480p", 0.8, (3, 38)),
    "image": ("image", 0.5, (0, 23)),
    "longvideo_s90": ("longvideo", 0.9, (11,)),
    "longvideo_s80": ("longvideo", 0.8, (19,)),
    "longvideo_s70": ("longvideo", 0.7, (2,)),
    "longvideo_s50": ("longvideo", 0.5, (5,)),
    # cumulative-mass selection with 512 text tokens: variable row lengths at full size
    "video720p_cdf_text": ("video720p", 0.8, (7,)),
    # 64-token blocks: 1,182 blocks per head (the mask kernel's wide-row path), two wavefronts per workgroup
    "video720p_b64": ("video720p", 0.8, (21,)),
    # 256-row Q blocks over 128-row K/V blocks: eight wavefronts per workgroup, rectangular 296 x 591 mask
    "video720p_q256_k128": ("video720p", 0.8, (33,)),
    # the remaining shapes of the kernels at the size the work tables and rings are built for:
    # head_dim 64 (one or two direct-to-LDS loads per wavefront and part), token-major q/k/v/o
    # (strided gathers and scatter over 75,600 tokens), 64-row K/V blocks under 128- and 256-row Q blocks
    "video720p_d64": ("video720p", 0.8, (12,)),
    "video720p_bnhd": ("video720p", 0.8, (29,)),
    "video720p_q128_k64": ("video720p", 0.8, (5,)),
    "video720p_q256_k64": ("video720p", 0.8, (36,)),
    # the largest block counts a plan accepts (2,048 rows and columns of the block mask): the mask kernel's
    # score strip at its full width (128 KiB of LDS), the longest lists, the largest work tables
    "limit_2048_blocks_b128": ("limit_2048_blocks_b128", 0.9, (0, 1)),
    "limit_2048_blocks_b64": ("limit_2048_blocks_b64", 0.9, (1,)),
}
# synthetic grids that exist only to reach the limits of the plan (not workloads of the paper)
LIMIT_WORKLOADS = {
    "limit_2048_blocks_b128": inputs.Workload("limit_2048_blocks_b128", 6, 1, 2, 64, 64, 64, 64, 128, 0.9, 1, 0.3),
    "limit_2048_blocks_b64": inputs.Workload("limit_2048_blocks_b64", 7, 1, 2, 128, 32, 64, 64, 64, 0.9, 1, 0.3),
}
EXTRA = {"video720p_cdf_text": dict(cdf_threshold=0.9, text_tokens=512), "video720p_b64": dict(block=64),
         "video720p_q256_k128": dict(block=256, block_k=128), "video720p_d64": dict(head_dim=64),
         "video720p_bnhd": dict(qkv_layout=rf2.RF2_LAYOUT_BNHD), "video720p_q128_k64": dict(block_k=64),
         "video720p_q256_k64": dict(block=256, block_k=64)}
# every Q block of this head of this case is checked against the oracle (the others: sampled blocks)
COMPLETE_HEAD = {"video720p": 17}


class Big:
    """One full-size case: plan, inputs as the oracle reads them (head-major) and as the library
    is given them (`dev`: token-major when the plan says so), buffers, oracle intermediates."""

    def o_head(self, h):
        o = self.buf["o"]
        return o[0, :, h] if self.plan.cfg.qkv_layout == rf2.RF2_LAYOUT_BNHD else o[0, h]


@pytest.fixture(scope="module", params=list(CASES), ids=list(CASES))
def big(request):
    name, s, heads = CASES[request.param]
    wl = inputs.WORKLOADS.get(name) or LIMIT_WORKLOADS[name]
    extra = dict(EXTRA.get(request.param, {}))
    import dataclasses
    for field in ("text_tokens", "block", "head_dim"):
        if field in extra:
            wl = dataclasses.replace(wl, **{field: extra.pop(field)})
    print(f"\n[case] {request.param}: {wl.name} N={wl.N} heads={wl.heads} d={wl.head_dim} sparsity={s} "
          f"sampled heads {heads} {extra}", flush=True)
    g = Big()
    g.name, g.wl = request.param, wl
    g.plan = plan = hp.make_plan(wl, sparsity=s, **extra)
    g.qkv = q, k, v = inputs.make_qkv(wl, device=DEV)
    g.dev = g.qkv
    if plan.cfg.qkv_layout == rf2.RF2_LAYOUT_BNHD:
        g.dev = tuple(x.transpose(1, 2).contiguous() for x in g.qkv)
    g.buf = buf = plan.alloc(DEV)
    plan.layer(*g.dev, buf)
    torch.cuda.synchronize()
    i, c = plan.info, plan.cfg
    rng = np.random.default_rng(wl.index)
    g.blocks = sorted({0, i.n_blocks - 1, *rng.integers(0, i.n_blocks, 4).tolist()} |
                      ({i.sink_block_begin, i.n_blocks - 2} if i.sink_block_end > i.sink_block_begin else set()))
    g.ref = ref = {}
    for h in heads:
        Q, K, V = (hp.f64(x[0, h].cpu()) for x in (q, k, v))
        perm = orc.perm_table(c.T, c.H, c.W, i.wt, i.wh, i.ww, c.sink_frames, bool(c.sink_at_end), c.text_tokens)
        Qp, Kp, Vp = orc.permute(Q, perm), orc.permute(K, perm), orc.permute(V, perm)
        qbar, kbar = orc.pool_blocks(Qp, c.block), orc.pool_blocks(Kp, i.block_k)
        S_hat = orc.block_scores(qbar, kbar)
        rows, cols = (i.sink_block_begin, i.sink_block_end), (i.sink_block_begin_k, i.sink_block_end_k)
        if c.select_mode == 1:
            M, gap = orc.select_blocks_cdf(S_hat, float(c.cdf_threshold), c.head_dim, *rows, cols)
        else:
            M = orc.select_blocks(S_hat, i.k_sel, *rows, cols)
            gap = orc.selection_gap(S_hat, i.k_sel, *rows, cols)
        ref[h] = dict(perm=perm, Qp=Qp, Kp=Kp, Vp=Vp, qbar=qbar, kbar=kbar, S_hat=S_hat, M=M, gap=gap)
        print(f"[oracle] head {h} done", flush=True)
    yield g
    plan.close()


def test_permutation_and_pooling(big):
    plan, (q, k, v), buf, ref = big.plan, big.qkv, big.buf, big.ref
    N = plan.info.N
    for h, r in ref.items():
        qp = inputs.bf16_bits(buf["qp"][0, h])
        kp = hp.kp_to_rows(inputs.bf16_bits(buf["kp"][0, h]))
        vp = hp.vp_to_rows(inputs.bf16_bits(buf["vp"][0, h]))
        for got, src in ((qp, q), (kp, k), (vp, v)):
            assert np.array_equal(got[:N], inputs.bf16_bits(src[0, h])[r["perm"]])
            assert (got[N:] == 0).all()
        for name in ("qbar", "kbar"):
            assert np.abs(buf[name][0, h].double().cpu().numpy() - r[name]).max() < (4e-6 if plan.cfg.block == 256 else 2e-6)


def test_block_mask(big):
    plan, buf, ref = big.plan, big.buf, big.ref
    i = plan.info
    Tq, Tb = i.n_blocks, i.n_blocks_k             # rows and columns of the mask (Tb: K blocks)
    sink = np.zeros(Tq, dtype=bool)
    sink[i.sink_block_begin:i.sink_block_end] = True
    # properties over ALL heads: row counts, ascending in-range lists, sink columns present
    cdf = plan.cfg.select_mode == 1
    cnt = buf["blk_cnt"][0].cpu().numpy()
    idx = buf["blk_idx"][0].cpu().numpy()
    assert (cnt[:, sink] == Tb).all()
    if cdf:
        n_sink = i.sink_block_end_k - i.sink_block_begin_k
        assert (cnt[:, ~sink] > n_sink).all() and (cnt[:, ~sink] <= Tb).all()
        print(f"[mask] cumulative-mass rows keep {cnt[:, ~sink].min()}..{cnt[:, ~sink].max()} blocks, "
              f"mean {cnt[:, ~sink].mean():.1f} of {Tb}")
    else:
        assert (cnt[:, ~sink] == i.k_row).all()
    rows = idx[:, ~sink, :]
    if i.k_row < Tb:
        assert (np.diff(rows, axis=-1) > 0).all() and rows.min() >= 0 and rows.max() < Tb
        n_sink = i.sink_block_end_k - i.sink_block_begin_k
        if n_sink:                                   # sink blocks sit at the end of the sequence: last entries of each list
            assert (rows[..., -n_sink:] == np.arange(i.sink_block_begin_k, i.sink_block_end_k)).all()
    near = differing = 0
    sink_cols = np.zeros(Tb, dtype=bool)
    sink_cols[i.sink_block_begin_k:i.sink_block_end_k] = True
    for h, r in ref.items():
        M = hp.gpu_lists_to_mask(buf["blk_idx"][0, h], buf["blk_cnt"][0, h], Tq, Tb)
        clear = r["gap"] > (hp.CDF_TIE if cdf else hp.TIE_GAP)
        near += int((~clear & ~sink).sum())
        assert np.array_equal(M[clear], r["M"][clear])
        assert (np.abs(M.sum(1) - r["M"].sum(1)) <= (1 if cdf else 0)).all()
        differing += hp.check_exempt_rows(M, r["M"], r["S_hat"], ~clear & ~sink, sink_cols,
                                          **(dict(d=plan.cfg.head_dim) if cdf else dict(k_sel=i.k_sel)))
    print(f"[mask] near-tie rows exempted: {near} of {len(ref) * int((~sink).sum())} "
          f"({differing} of them differ from the oracle's, all within the tie)")


def test_attention_on_sampled_blocks(big):
    plan, buf, ref = big.plan, big.buf, big.ref
    i, b = plan.info, plan.cfg.block
    worst = (0.0, 0.0)
    for h, r in ref.items():
        M = hp.gpu_lists_to_mask(buf["blk_idx"][0, h], buf["blk_cnt"][0, h], i.n_blocks, i.n_blocks_k)   # the mask the GPU used
        complete = COMPLETE_HEAD.get(big.name) == h
        blocks = list(range(i.n_blocks)) if complete else big.blocks
        want = orc.block_sparse_attention(r["Qp"], r["Kp"], r["Vp"], M, b, q_blocks=blocks, bk=i.block_k)
        got = hp.f64(buf["op"][0, h].cpu())[:i.N]
        rows = ~np.isnan(want[:, 0])
        err = np.abs(got[rows] - want[rows])
        assert err.max() <= hp.ATTN_MAX_ABS and err.mean() <= hp.ATTN_MEAN_ABS, (h, err.max(), err.mean())
        worst = (max(worst[0], err.max()), max(worst[1], err.mean()))
        # the unpermuted output is a bit-exact scatter of the permuted one
        o_bits = inputs.bf16_bits(big.o_head(h))
        assert np.array_equal(o_bits[r["perm"]], inputs.bf16_bits(buf["op"][0, h])[:i.N])
        print(f"[attention] head {h}: " + (f"all {i.n_blocks} Q blocks" if complete else f"Q blocks {blocks}")
              + f": max abs {err.max():.2e}, mean abs {err.mean():.2e}", flush=True)
    print(f"[attention] worst: max abs {worst[0]:.2e}, mean abs {worst[1]:.2e}")


def test_constant_values_give_constant_output(big):
    """V == 1 everywhere must give O == 1 on every row of every head (probabilities sum to one)."""
    plan, (q, k, v), buf = big.plan, big.dev, big.buf
    ones = torch.ones_like(v)
    plan.rf2_permute(q, k, ones, buf["qp"], buf["kp"], buf["vp"])
    plan.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"], buf["blk_cnt"], buf["op"])
    plan.rf2_unpermute(buf["op"], buf["o"])
    torch.cuda.synchronize()
    dev = (buf["o"].float() - 1.0).abs().max().item()
    assert dev <= 2 ** -7, dev                      # bf16 rounding of the probabilities and of the output


def test_maximum_number_of_heads():
    """B x Hh = 65,535, the most a plan accepts (the second grid dimension of the permutation and mask
    launches): five seeded heads repeated 13,107 times.  The five are checked against the oracle; every
    repetition must equal the first one bit for bit (same inputs, deterministic kernels)."""
    base = inputs.Workload("limit_heads", 8, 1, 5, 64, 8, 8, 8, 64, 0.5, 1, 0.3)
    reps = 13107
    wl = inputs.Workload("limit_heads", 8, 1, base.heads * reps, 64, 8, 8, 8, 64, 0.5, 1, 0.3)
    assert wl.heads == 65535
    q5, k5, v5 = inputs.make_qkv(base)
    plan = hp.make_plan(wl)
    dev = [x.to(DEV).repeat(1, reps, 1, 1) for x in (q5, k5, v5)]
    buf = plan.alloc(DEV)
    o = plan.layer_fused(*dev, buf)
    torch.cuda.synchronize()
    i = plan.info
    for name in ("o", "blk_idx", "blk_cnt", "qbar", "kbar"):
        t = buf[name][0]
        first = t[:base.heads]
        assert torch.equal(t.reshape(reps, *first.shape), first.expand(reps, *first.shape)), name
    for h in range(base.heads):
        Q, K, V = (hp.f64(x[0, h]) for x in (q5, k5, v5))
        r = orc.layer(Q, K, V, T=wl.T, H=wl.H, W=wl.W, block=wl.block, sparsity=wl.sparsity,
                      sink_frames=wl.sink_frames, window=(i.wt, i.wh, i.ww))
        for hh in (h, wl.heads - base.heads + h):           # first and last repetition
            M = hp.gpu_lists_to_mask(buf["blk_idx"][0, hh], buf["blk_cnt"][0, hh], i.n_blocks)
            firm = r["gap"] > hp.TIE_GAP
            assert np.array_equal(M[firm], r["M"][firm]), hh
            want = r["O"] if np.array_equal(M, r["M"]) else orc.unpermute(
                orc.block_sparse_attention(r["Qp"], r["Kp"], r["Vp"], M, wl.block), r["perm"])
            err = np.abs(hp.f64(o[0, hh].cpu()) - want)
            assert err.max() <= hp.ATTN_MAX_ABS and err.mean() <= hp.ATTN_MEAN_ABS, (hh, err.max(), err.mean())
    plan.close()
