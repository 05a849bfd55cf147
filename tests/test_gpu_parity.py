"""GPU parity: every stage of the HIP path vs. the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import rf2_oracle as orc
from paper_2512_24086_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda"

SMALL = {
    # name: (workload, plan overrides)
    "tiny": (inputs.WORKLOADS["tiny"], {}),
    "tiny_sink_front": (inputs.WORKLOADS["tiny"], dict(sink_at_end=0)),
    "tiny_dense": (inputs.WORKLOADS["tiny"], dict(sparsity=0.0)),
    "ragged_d128_b128": (inputs.Workload("ragged", 6, 1, 3, 128, 5, 10, 13, 128, 0.5, 1, 0.3), {}),
    "ragged_d128_b64": (inputs.Workload("ragged2", 7, 1, 2, 128, 4, 9, 11, 64, 0.6, 1, 0.3), dict(window=(2, 4, 4))),
    "ragged_d64_b128": (inputs.Workload("ragged3", 8, 1, 2, 64, 3, 12, 15, 128, 0.4, 0, 0.3), {}),
    "image_small": (inputs.Workload("img", 9, 1, 2, 128, 1, 40, 36, 128, 0.5, 0, 0.3), {}),
    "one_block": (inputs.Workload("one", 10, 1, 1, 128, 1, 5, 7, 128, 0.5, 0, 0.3), {}),
    "row_incl_sink": (inputs.WORKLOADS["tiny"], dict(budget_mode=1, sparsity=0.6)),
    # text tokens appended to the video tokens (ragged last block, always-dense tail)
    "tiny_text": (inputs.Workload("tinytext", 13, 1, 2, 64, 6, 16, 16, 64, 0.5, 1, 0.3, text_tokens=40), {}),
    "image_text_d128": (inputs.Workload("imgtext", 14, 1, 2, 128, 1, 40, 36, 128, 0.5, 0, 0.3, text_tokens=77), {}),
    # cumulative-mass selection: rows of different lengths
    "tiny_cdf": (inputs.WORKLOADS["tiny"], dict(cdf_threshold=0.7)),
    "ragged_cdf_d128": (inputs.Workload("raggedcdf", 15, 1, 3, 128, 5, 10, 13, 128, 0.5, 1, 0.3, text_tokens=9),
                        dict(cdf_threshold=0.9)),
    # different block sizes for Q and K (rectangular block mask)
    "q128_k64": (inputs.Workload("q128k64", 16, 1, 2, 128, 5, 10, 13, 128, 0.5, 1, 0.3), dict(block_k=64)),
    "q64_k128_d64": (inputs.Workload("q64k128", 17, 1, 2, 64, 6, 16, 16, 64, 0.5, 1, 0.3), dict(block_k=128)),
    "q256_k128": (inputs.Workload("q256k128", 18, 1, 2, 128, 7, 12, 16, 256, 0.6, 1, 0.3, text_tokens=30),
                  dict(block_k=128)),
    "q256_k64_d64": (inputs.Workload("q256k64", 19, 1, 2, 64, 5, 12, 16, 256, 0.5, 1, 0.3), dict(block_k=64)),
    # combinations: fewer tokens than one Q block; cumulative-mass rows over a rectangular mask with text tokens
    "q256_single_block": (inputs.Workload("q256one", 20, 1, 1, 128, 1, 9, 11, 256, 0.5, 0, 0.3), dict(block_k=128)),
    "q256_k128_cdf_text": (inputs.Workload("q256cdf", 21, 1, 2, 128, 6, 12, 16, 256, 0.5, 1, 0.3, text_tokens=70),
                           dict(block_k=128, cdf_threshold=0.8)),
    # two sink frames (2-D windows frame by frame), a window that does not divide the body; third budget reading
    "two_sink_frames": (inputs.Workload("sink2", 24, 1, 2, 64, 7, 10, 13, 64, 0.3, 2, 0.3), dict(window=(2, 4, 8))),
    "row_plus_sink": (inputs.WORKLOADS["tiny"], dict(budget_mode=2, sparsity=0.7)),
    "q64_k128_sink_front": (inputs.Workload("q64front", 22, 1, 2, 128, 4, 9, 11, 64, 0.6, 1, 0.3),
                            dict(block_k=128, sink_at_end=0)),
}


@pytest.fixture(scope="module", params=list(SMALL), ids=list(SMALL))
def case(request):
    wl, over = SMALL[request.param]
    print(f"\n[case] {request.param}: {wl}", flush=True)
    plan = hp.make_plan(wl, **over)
    q, k, v = inputs.make_qkv(wl)
    qd, kd, vd = (x.to(DEV) for x in (q, k, v))
    buf = plan.alloc(DEV, dense_mask=True, scores=True, lse=True)
    for t in buf.values():
        t.fill_(0) if t.dtype != torch.bfloat16 else t.copy_(torch.full_like(t, float("nan")))
    plan.layer(qd, kd, vd, buf)
    torch.cuda.synchronize()
    ref = [hp.oracle_layer(wl, q, k, v, h, plan) for h in range(wl.heads)]
    yield wl, plan, (q, k, v), (qd, kd, vd), buf, ref
    plan.close()


def test_permute_is_bit_exact(case):
    wl, plan, (q, k, v), _, buf, ref = case
    N, Np = plan.info.N, plan.info.N_pad
    for h in range(wl.heads):
        for name, src in (("qp", q), ("kp", k)):
            got = inputs.bf16_bits(buf[name][0, h])
            if name == "kp":
                got = hp.kp_to_rows(got)
            want = inputs.bf16_bits(src[0, h])[ref[h]["perm"]]
            assert np.array_equal(got[:N], want), name
            assert (got[N:] == 0).all(), "padding rows must be zero"
        got_v = hp.vp_to_rows(inputs.bf16_bits(buf["vp"][0, h]))
        assert np.array_equal(got_v[:N], inputs.bf16_bits(v[0, h])[ref[h]["perm"]])
        assert (got_v[N:] == 0).all()


def test_block_means(case):
    wl, plan, _, _, buf, ref = case
    for h in range(wl.heads):
        for name in ("qbar", "kbar"):
            got = buf[name][0, h].double().cpu().numpy()
            # fp32 sum of <=128 (256 for the largest Q block) bf16 values of magnitude ~1, then one division
            assert np.abs(got - ref[h][name]).max() < (4e-6 if plan.cfg.block == 256 else 2e-6), name


def test_scores_and_block_mask(case):
    wl, plan, _, _, buf, ref = case
    i = plan.info
    Tb, Tk = i.n_blocks, i.n_blocks_k             # rows (Q blocks) and columns (K blocks) of the mask
    near_ties = differing = 0
    for h in range(wl.heads):
        S = buf["scores"][0, h].double().cpu().numpy()
        assert np.abs(S - ref[h]["S_hat"]).max() < 1e-4          # fp32 dot products of length d, |S| ~ 10
        M = hp.gpu_lists_to_mask(buf["blk_idx"][0, h], buf["blk_cnt"][0, h], Tb, Tk)
        assert np.array_equal(M, buf["mask_dense"][0, h].cpu().numpy().astype(bool)), "list and dense mask disagree"
        cnt = buf["blk_cnt"][0, h].cpu().numpy()
        sink = np.zeros(Tb, dtype=bool)
        sink[i.sink_block_begin:i.sink_block_end] = True
        sink_cols = np.zeros(Tk, dtype=bool)
        sink_cols[i.sink_block_begin_k:i.sink_block_end_k] = True
        cdf = plan.cfg.select_mode == 1
        assert (cnt[sink] == Tk).all() and M[:, sink_cols].all() and M[sink].all()
        clear = ref[h]["gap"] > (hp.CDF_TIE if cdf else hp.TIE_GAP)
        near_ties += int((~clear & ~sink).sum())
        assert np.array_equal(M[clear], ref[h]["M"][clear]), "mask differs on a row with a clear boundary"
        differing += hp.check_exempt_rows(M, ref[h]["M"], ref[h]["S_hat"], ~clear & ~sink, sink_cols,
                                          **(dict(d=wl.head_dim) if cdf else dict(k_sel=i.k_sel)))
        if cdf:                                     # a near-tie row may be one column longer or shorter
            assert (cnt[~sink] == M[~sink].sum(1)).all() and (np.abs(M.sum(1) - ref[h]["M"].sum(1)) <= 1).all()
            if (~sink).sum() >= 16:
                assert len(set(cnt[~sink])) > 1, "cumulative-mass rows should differ in length on these inputs"
        else:
            assert (cnt[~sink] == i.k_row).all()
            assert (M.sum(1) == ref[h]["M"].sum(1)).all()
    print(f"[mask] near-tie rows exempted: {near_ties} ({differing} of them differ from the oracle's, all within the tie)")


def test_attention_with_oracle_mask(case):
    """Feeds the ORACLE's block lists to the kernel, isolating the attention arithmetic."""
    wl, plan, _, _, buf, ref = case
    i = plan.info
    idx, cnt = hp.lists_to_device([r["M"] for r in ref], i.k_row, i.n_blocks, DEV)
    op = torch.full_like(buf["op"], float("nan"))
    lse = torch.zeros_like(buf["lse"])
    plan.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], idx, cnt, op, lse)
    torch.cuda.synchronize()
    for h in range(wl.heads):
        got = hp.f64(op[0, h])[:i.N]
        err = np.abs(got - ref[h]["Op"])
        assert err.max() <= hp.ATTN_MAX_ABS and err.mean() <= hp.ATTN_MEAN_ABS, (err.max(), err.mean())
        got_lse = lse[0, h, :i.N].double().cpu().numpy()
        assert np.abs(got_lse - ref[h]["lse"]).max() < 2e-3


def test_whole_layer_and_unpermute(case):
    wl, plan, _, _, buf, ref = case
    i = plan.info
    for h in range(wl.heads):
        op_bits = inputs.bf16_bits(buf["op"][0, h])[:i.N]
        o_bits = inputs.bf16_bits(buf["o"][0, h])
        assert np.array_equal(o_bits[ref[h]["perm"]], op_bits), "unpermute must be a bit-exact scatter"
        M = hp.gpu_lists_to_mask(buf["blk_idx"][0, h], buf["blk_cnt"][0, h], i.n_blocks, i.n_blocks_k)
        if np.array_equal(M, ref[h]["M"]):
            want = ref[h]["O"]
        else:                                  # near-tie rows chose differently: oracle attention on the GPU's mask
            Op = orc.block_sparse_attention(ref[h]["Qp"], ref[h]["Kp"], ref[h]["Vp"], M, plan.cfg.block,
                                            bk=plan.info.block_k)
            want = orc.unpermute(Op, ref[h]["perm"])
        err = np.abs(hp.f64(buf["o"][0, h]) - want)
        assert err.max() <= hp.ATTN_MAX_ABS and err.mean() <= hp.ATTN_MEAN_ABS, (err.max(), err.mean())


def test_round_trip_is_identity():
    wl = inputs.WORKLOADS["tiny"]
    plan = hp.make_plan(wl)
    q, k, v = (x.to(DEV) for x in inputs.make_qkv(wl))
    buf = plan.alloc(DEV)
    plan.rf2_permute(q, k, v, buf["qp"], buf["kp"], buf["vp"])          # no pooling requested
    plan.rf2_unpermute(buf["qp"], buf["o"])          # qp is row-major like op
    torch.cuda.synchronize()
    assert torch.equal(buf["o"].view(torch.int16), q.view(torch.int16))
    plan.close()


def test_dense_layer_is_independent_of_the_permutation():
    """At sparsity 0 the layer is plain attention: window shape and sink placement cannot matter."""
    wl = inputs.Workload("inv", 11, 1, 2, 128, 4, 9, 11, 128, 0.0, 1, 0.3)
    q, k, v = inputs.make_qkv(wl)
    qd, kd, vd = (x.to(DEV) for x in (q, k, v))
    outs = []
    for over in (dict(), dict(window=(1, 3, 5), sink_at_end=0), dict(window=(4, 9, 11), sink_frames=0)):
        plan = hp.make_plan(wl, **over)
        buf = plan.alloc(DEV)
        outs.append(hp.f64(plan.layer(qd, kd, vd, buf)))
        torch.cuda.synchronize()
        plan.close()
    dense = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(hp.f64(q)), torch.from_numpy(hp.f64(k)), torch.from_numpy(hp.f64(v))).numpy()
    for o in outs:
        err = np.abs(o - dense)
        assert err.max() <= hp.ATTN_MAX_ABS and err.mean() <= hp.ATTN_MEAN_ABS


def test_fused_inverse_permutation_matches_separate_calls(case):
    """rf2_block_sparse_attn_unpermuted == rf2_block_sparse_attn followed by rf2_unpermute, bit for bit."""
    wl, plan, _, _, buf, _ = case
    i = plan.info
    o2 = torch.full_like(buf["o"], float("nan"))
    lse2 = torch.full((wl.batch, wl.heads, i.N), float("nan"), dtype=torch.float32, device=DEV)
    plan.rf2_block_sparse_attn_unpermuted(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"], buf["blk_cnt"], o2, lse2)
    torch.cuda.synchronize()
    assert torch.equal(o2.view(torch.int16), buf["o"].view(torch.int16))
    perm, _ = plan.rf2_plan_perm()
    want_lse = buf["lse"][:, :, :i.N].cpu().numpy()
    got_lse = lse2.cpu().numpy()
    assert np.array_equal(got_lse[:, :, perm], want_lse)


def test_repeated_calls_are_bit_identical_and_streams_are_honoured():
    """No atomics anywhere: two runs give the same bits; work goes to the stream that is passed."""
    wl = inputs.WORKLOADS["tiny"]
    plan = hp.make_plan(wl)
    q, k, v = (x.to(DEV) for x in inputs.make_qkv(wl))
    buf1, buf2 = plan.alloc(DEV), plan.alloc(DEV)
    plan.layer(q, k, v, buf1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.layer_fused(q, k, v, buf2, stream=side)
    side.synchronize()
    torch.cuda.synchronize()
    for name in ("qp", "kp", "vp", "blk_idx", "blk_cnt", "o"):
        assert torch.equal(buf1[name].view(torch.int16) if buf1[name].dtype == torch.bfloat16 else buf1[name],
                           buf2[name].view(torch.int16) if buf2[name].dtype == torch.bfloat16 else buf2[name]), name
    assert torch.equal(buf1["qbar"], buf2["qbar"]) and torch.equal(buf1["kbar"], buf2["kbar"])
    plan.close()


def test_device_calls_reject_missing_arguments():
    wl = inputs.WORKLOADS["tiny"]
    plan = hp.make_plan(wl)
    buf = plan.alloc(DEV)
    q, k, v = (x.to(DEV) for x in inputs.make_qkv(wl))
    from paper_2512_24086_amd import rf2
    with pytest.raises(rf2.Rf2Error) as e:
        plan.rf2_permute(q, k, None, buf["qp"], buf["kp"], buf["vp"])
    assert e.value.code == rf2.RF2_ERR_INVALID_ARG
    with pytest.raises(rf2.Rf2Error):
        plan.rf2_permute(q, k, v, buf["qp"], buf["kp"], buf["vp"], buf["qbar"], None)    # means come in pairs
    with pytest.raises(rf2.Rf2Error):
        plan.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], None, buf["blk_cnt"], buf["op"])
    with pytest.raises(rf2.Rf2Error):
        plan.rf2_block_sparse_attn_unpermuted(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"], buf["blk_cnt"], None)
    with pytest.raises(rf2.Rf2Error):
        plan.rf2_predict_mask(buf["qbar"], None, buf["blk_idx"], buf["blk_cnt"])
    with pytest.raises(rf2.Rf2Error):
        plan.rf2_unpermute(None, buf["o"])
    plan.close()


def test_calls_made_under_another_device_are_rejected():
    """A plan computes on the device it was made on.  The box has one GPU, so the mismatch is staged from
    the host: the plan's recorded device number is changed in place (no launch happens while it is wrong)."""
    import ctypes as C
    from paper_2512_24086_amd import rf2
    wl = inputs.WORKLOADS["tiny"]
    plan = hp.make_plan(wl)
    buf = plan.alloc(DEV)
    q, k, v = (x.to(DEV) for x in inputs.make_qkv(wl))
    # struct rf2_plan starts with {rf2_config cfg; rf2_info info; int device; ...} (csrc/rf2_internal.h)
    off = -(-C.sizeof(rf2.rf2_config) // 8) * 8 + C.sizeof(rf2.rf2_info)
    device = C.c_int.from_address(plan._h.value + off)
    assert device.value == torch.cuda.current_device()
    device.value += 1
    try:
        calls = (lambda: plan.rf2_permute(q, k, v, buf["qp"], buf["kp"], buf["vp"], buf["qbar"], buf["kbar"]),
                 lambda: plan.rf2_predict_mask(buf["qbar"], buf["kbar"], buf["blk_idx"], buf["blk_cnt"]),
                 lambda: plan.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"], buf["blk_cnt"], buf["op"]),
                 lambda: plan.rf2_block_sparse_attn_unpermuted(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"],
                                                               buf["blk_cnt"], buf["o"]),
                 lambda: plan.rf2_unpermute(buf["op"], buf["o"]))
        for call in calls:
            with pytest.raises(rf2.Rf2Error) as e:
                call()
            assert e.value.code == rf2.RF2_ERR_INVALID_ARG
    finally:
        device.value -= 1
    plan.layer(q, k, v, buf)                       # and the plan works again on its own device
    torch.cuda.synchronize()
    plan.close()


def test_empty_and_corrupt_lists_do_not_fault():
    """Counts of zero give zero rows; out-of-range entries are clamped (wrong values, never a fault)."""
    wl = inputs.WORKLOADS["tiny"]
    plan = hp.make_plan(wl)
    q, k, v = (x.to(DEV) for x in inputs.make_qkv(wl))
    buf = plan.alloc(DEV, lse=True)
    plan.layer(q, k, v, buf)
    cnt = torch.zeros_like(buf["blk_cnt"])
    plan.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"], cnt, buf["op"], buf["lse"])
    torch.cuda.synchronize()
    assert (buf["op"].float() == 0).all() and torch.isinf(buf["lse"]).all()
    bad = torch.full_like(buf["blk_idx"], 10 ** 6)
    bad[..., 0] = -5
    plan.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], bad, torch.full_like(cnt, plan.info.k_row), buf["op"])
    torch.cuda.synchronize()
    assert torch.isfinite(buf["op"].float()).all()
    plan.close()


@pytest.mark.parametrize("scale", [8.0, 32.0])
def test_large_logits_take_the_reference_reset_path(scale):
    """Logits hundreds of log2 units apart between blocks: the exponentials' reference point must be
    re-based (overflow of a unit's row sum), and the result must still match the oracle."""
    wl = inputs.Workload("hot", 12, 1, 2, 128, 4, 12, 16, 128, 0.4, 1, 0.3)
    plan = hp.make_plan(wl)
    q, k, v = inputs.make_qkv(wl)
    q = (q.float() * scale).to(torch.bfloat16)            # exact in bf16 (power of two)
    k = (k.float() * scale).to(torch.bfloat16)
    buf = plan.alloc(DEV, lse=True)
    o = plan.layer(q.to(DEV), k.to(DEV), v.to(DEV), buf)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
    for h in range(wl.heads):
        ref = hp.oracle_layer(wl, q, k, v, h, plan)
        M = hp.gpu_lists_to_mask(buf["blk_idx"][0, h], buf["blk_cnt"][0, h], plan.info.n_blocks, plan.info.n_blocks_k)
        want = ref["O"]
        if not np.array_equal(M, ref["M"]):
            Op = orc.block_sparse_attention(ref["Qp"], ref["Kp"], ref["Vp"], M, plan.cfg.block, bk=plan.info.block_k)
            want = orc.unpermute(Op, ref["perm"])
        err = np.abs(hp.f64(o[0, h]) - want)
        assert err.max() <= hp.ATTN_MAX_ABS and err.mean() <= hp.ATTN_MEAN_ABS, (scale, err.max(), err.mean())
    plan.close()


@pytest.mark.parametrize("name", ["tiny", "ragged_d128_b128"])
def test_token_major_layout_gives_identical_results(name):
    """q, k, v, o held as [B, N, Hh, d]: every intermediate and the output are bit-identical to the
    head-major run (the layout only changes the addresses of the gathers and of the final scatter)."""
    from paper_2512_24086_amd import rf2
    wl, over = SMALL[name]
    q, k, v = (x.to(DEV) for x in inputs.make_qkv(wl))
    plan_a = hp.make_plan(wl, **over)
    plan_b = hp.make_plan(wl, qkv_layout=rf2.RF2_LAYOUT_BNHD, **over)
    buf_a, buf_b = plan_a.alloc(DEV), plan_b.alloc(DEV)
    qt, kt, vt = (x.transpose(1, 2).contiguous() for x in (q, k, v))
    plan_a.layer(q, k, v, buf_a)
    plan_b.layer(qt, kt, vt, buf_b)
    torch.cuda.synchronize()
    assert buf_b["o"].shape == (wl.batch, wl.N, wl.heads, wl.head_dim)
    for n in ("qp", "kp", "vp", "op"):
        assert torch.equal(buf_a[n].view(torch.int16), buf_b[n].view(torch.int16)), n
    assert torch.equal(buf_a["qbar"], buf_b["qbar"]) and torch.equal(buf_a["blk_idx"], buf_b["blk_idx"])
    assert torch.equal(buf_a["o"].view(torch.int16), buf_b["o"].transpose(1, 2).contiguous().view(torch.int16))
    o_fused = torch.full_like(buf_b["o"], float("nan"))
    plan_b.rf2_block_sparse_attn_unpermuted(buf_b["qp"], buf_b["kp"], buf_b["vp"], buf_b["blk_idx"], buf_b["blk_cnt"],
                                            o_fused)
    torch.cuda.synchronize()
    assert torch.equal(o_fused.view(torch.int16), buf_b["o"].view(torch.int16))
    plan_a.close()
    plan_b.close()


@pytest.mark.parametrize("layout", ["BHND", "BNHD"])
def test_batch_of_two(layout):
    """B = 2, three heads, ragged last block: every (batch, head) slice against the oracle, in both
    memory orders, through the fused and the unfused exit."""
    from paper_2512_24086_amd import rf2
    wl = inputs.Workload("batch2", 23, 2, 3, 128, 4, 9, 11, 128, 0.5, 1, 0.3, text_tokens=5)
    q, k, v = inputs.make_qkv(wl)
    assert not torch.equal(q[0], q[1])
    token_major = layout == "BNHD"
    plan = hp.make_plan(wl, qkv_layout=rf2.RF2_LAYOUT_BNHD if token_major else rf2.RF2_LAYOUT_BHND)
    dev = [x.to(DEV) for x in (q, k, v)]
    if token_major:
        dev = [x.transpose(1, 2).contiguous() for x in dev]
    buf = plan.alloc(DEV, lse=True)
    o_fused = plan.layer_fused(*dev, buf).clone()           # inverse permutation in the attention epilogue
    buf["o"].fill_(float("nan"))
    plan.layer(*dev, buf)                                   # attention into op, then rf2_unpermute
    torch.cuda.synchronize()
    assert torch.equal(o_fused.view(torch.int16), buf["o"].view(torch.int16))
    o = o_fused.transpose(1, 2) if token_major else o_fused
    i = plan.info
    for b in range(wl.batch):
        for h in range(wl.heads):
            Q, K, V = (hp.f64(x[b, h]) for x in (q, k, v))
            r = orc.layer(Q, K, V, T=wl.T, H=wl.H, W=wl.W, block=wl.block, sparsity=wl.sparsity,
                          sink_frames=wl.sink_frames, window=(i.wt, i.wh, i.ww), text_tokens=wl.text_tokens)
            M = hp.gpu_lists_to_mask(buf["blk_idx"][b, h], buf["blk_cnt"][b, h], i.n_blocks)
            firm = r["gap"] > hp.TIE_GAP
            assert np.array_equal(M[firm], r["M"][firm]), (b, h)
            sink_cols = np.zeros(i.n_blocks_k, dtype=bool)
            sink_cols[i.sink_block_begin_k:i.sink_block_end_k] = True
            hp.check_exempt_rows(M, r["M"], r["S_hat"], ~firm, sink_cols, k_sel=i.k_sel)
            if not np.array_equal(M, r["M"]):               # a near-tie row differs: compare on the GPU's own mask
                Qp, Kp, Vp = r["Qp"], r["Kp"], r["Vp"]
                want = orc.unpermute(orc.block_sparse_attention(Qp, Kp, Vp, M, wl.block), r["perm"])
            else:
                want = r["O"]
            err = np.abs(hp.f64(o[b, h]) - want)
            assert err.max() <= hp.ATTN_MAX_ABS and err.mean() <= hp.ATTN_MEAN_ABS, (b, h, err.max(), err.mean())
            assert np.array_equal(hp.f64(buf["qp"][b, h])[:wl.N], r["Qp"]), (b, h)
    plan.close()


def test_measured_peaks_are_plausible():
    """The measurement aid returns the MFMA-loop rate and the copy bandwidth of this GPU."""
    from paper_2512_24086_amd import rf2
    mfma, copy = rf2.rf2_measure_peaks()
    assert 500.0 < mfma <= 2600.0, mfma        # dense bf16 peak of the chip is 2.5 PFLOP/s
    assert 1000.0 < copy <= 8200.0, copy       # HBM3E peak is 8 TB/s


def test_workgroups_of_a_residue_class_share_an_xcd():
    """The attention kernel hands the workgroups g with equal g % 8 a contiguous range of a head's Q blocks,
    so that their K/V tiles meet in one L2: the classes must sit on eight different XCDs, every workgroup
    on the XCD of its class.  (Which XCD class 0 gets varies from launch to launch.)"""
    from paper_2512_24086_amd import rf2
    seen = set()
    for _ in range(3):
        agree, total, first = rf2.rf2_probe_xcd_mapping()
        assert total == 8192 and agree == total, (agree, total)
        assert 0 <= first < 8
        seen.add(first)
    print(f"[xcd] workgroup 0 ran on XCD {sorted(seen)} in three launches")


def test_sustained_mfma_rate_is_below_the_short_loop():
    """Pseudo-random operands under the power limit: a plausible rate, and not above the constant-operand loop."""
    from paper_2512_24086_amd import rf2
    short, _ = rf2.rf2_measure_peaks()
    sustained = rf2.rf2_measure_sustained_mfma(0.6)
    assert 300.0 < sustained <= short * 1.02, (sustained, short)
