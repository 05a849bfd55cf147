"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and its
host logic (config validation, sizes, permutation tables) agrees with the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import rf2_oracle as orc
from paper_2512_24086_amd import rf2
from paper_2512_24086_amd.inputs import WORKLOADS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rf2.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rf2_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = rf2.lib()
    names = declared_symbols()
    assert set(names) == set(rf2.SIGNATURES), "binding and header disagree on the entry points"
    for n in names:
        assert getattr(lib, n) is not None
    assert lib.rf2_version() >= 100
    assert lib.rf2_strerror(0) == b"ok" and b"invalid" in lib.rf2_strerror(-1)


def make_plan(**kw):
    base = dict(batch=1, heads=2, head_dim=64, T=6, H=16, W=16, block=64, sparsity=0.5, sink_frames=1)
    base.update(kw)
    return rf2.Plan(**base)


@pytest.mark.parametrize("bad", [
    dict(batch=0), dict(heads=0), dict(T=0), dict(sink_frames=6), dict(sink_frames=-1), dict(sparsity=1.0),
    dict(sparsity=-0.1), dict(sparsity=float("nan")), dict(budget_mode=3), dict(window=(0, 4, 4)),
    dict(window=(-1, 4, 4)), dict(sink_at_end=2), dict(qkv_layout=2), dict(qkv_layout=-1), dict(text_tokens=-1),
    dict(cdf_threshold=0.0), dict(cdf_threshold=1.0), dict(cdf_threshold=float("nan")),
])
def test_invalid_configs_are_rejected(bad):
    with pytest.raises(rf2.Rf2Error) as e:
        make_plan(**bad)
    assert e.value.code == rf2.RF2_ERR_INVALID_ARG


@pytest.mark.parametrize("bad", [dict(head_dim=96), dict(block=32), dict(T=4096, H=256, W=256),
                                 dict(text_tokens=5, sink_at_end=0),     # dense tokens in two separate runs
                                 dict(block=256), dict(block_k=256), dict(block_k=32), dict(block=256, block_k=256)])
def test_unsupported_configs_are_rejected(bad):
    with pytest.raises(rf2.Rf2Error) as e:
        make_plan(**bad)
    assert e.value.code == rf2.RF2_ERR_UNSUPPORTED


def test_null_arguments_are_rejected():
    lib = rf2.lib()
    assert lib.rf2_plan_create(None, None) == rf2.RF2_ERR_INVALID_ARG
    assert lib.rf2_plan_info(None, None) == rf2.RF2_ERR_INVALID_ARG
    assert lib.rf2_permute(*([None] * 10)) == rf2.RF2_ERR_INVALID_ARG
    assert lib.rf2_predict_mask(*([None] * 9)) == rf2.RF2_ERR_INVALID_ARG
    assert lib.rf2_block_sparse_attn(*([None] * 9)) == rf2.RF2_ERR_INVALID_ARG
    assert lib.rf2_unpermute(*([None] * 4)) == rf2.RF2_ERR_INVALID_ARG
    assert lib.rf2_measure_peaks(None, None, None) == rf2.RF2_ERR_INVALID_ARG
    out = C.c_double(0.0)
    assert lib.rf2_measure_sustained_mfma(C.c_double(1.0), None, None) == rf2.RF2_ERR_INVALID_ARG
    for bad_seconds in (0.0, -1.0, float("nan"), 31.0):
        assert lib.rf2_measure_sustained_mfma(C.c_double(bad_seconds), C.byref(out), None) == rf2.RF2_ERR_INVALID_ARG
    assert lib.rf2_probe_xcd_mapping(None, None, None, None) == rf2.RF2_ERR_INVALID_ARG
    # the allocation-free probe checks its sizes before it touches the device
    dummy = C.c_void_p(0x1000)
    assert lib.rf2_probe_xcd_mapping_static(C.c_int32(64), None, None) == rf2.RF2_ERR_INVALID_ARG
    assert lib.rf2_probe_xcd_mapping_static(C.c_int32(7), dummy, None) == rf2.RF2_ERR_INVALID_ARG
    assert lib.rf2_probe_xcd_mapping_static(C.c_int32(8193), dummy, None) == rf2.RF2_ERR_TOO_LARGE
    assert b"static device array" in lib.rf2_strerror(rf2.RF2_ERR_TOO_LARGE)
    assert lib.rf2_plan_destroy(None) == rf2.RF2_OK


@pytest.mark.parametrize("name", list(WORKLOADS))
def test_plan_sizes_and_tables_match_the_oracle(name):
    wl = WORKLOADS[name]
    for s in (wl.sweep or (wl.sparsity,)):
        p = make_plan(batch=wl.batch, heads=wl.heads, head_dim=wl.head_dim, T=wl.T, H=wl.H, W=wl.W,
                      block=wl.block, sparsity=s, sink_frames=wl.sink_frames)
        i = p.info
        Tb = orc.n_blocks(wl.N, wl.block)
        sb, se = orc.sink_block_range(wl.N, wl.H * wl.W, wl.block, wl.sink_frames, True)
        k_row, k_sel = orc.budget(Tb, se - sb, s)
        assert (i.N, i.n_blocks, i.N_pad) == (wl.N, Tb, Tb * wl.block)
        assert i.last_block_valid == wl.N - (Tb - 1) * wl.block
        assert (i.sink_block_begin, i.sink_block_end) == (sb, se)
        assert (i.k_row, i.k_sel) == (k_row, k_sel)
        assert i.kept_pairs_per_head == orc.kept_pairs(Tb, se - sb, k_row)
        assert abs(i.achieved_sparsity - (1 - i.kept_pairs_per_head / Tb ** 2)) < 1e-12
        assert (i.wt, i.wh, i.ww) == orc.default_window(wl.block, wl.T > 1)
    perm, inv = p.rf2_plan_perm()
    want = orc.perm_table(wl.T, wl.H, wl.W, i.wt, i.wh, i.ww, wl.sink_frames, True)
    assert np.array_equal(perm, want)                      # bit-exact index parity
    assert np.array_equal(inv, orc.inverse_table(want))
    p.close()


@pytest.mark.parametrize("case", [
    (5, 7, 9, (2, 4, 4), 1, 1), (5, 7, 9, (2, 4, 4), 1, 0), (5, 7, 9, (3, 2, 5), 0, 1), (4, 5, 3, (3, 2, 2), 2, 1),
    (1, 10, 13, (1, 8, 16), 0, 1), (7, 3, 5, (2, 2, 3), 3, 0),
])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_ragged_tables_and_budget_modes(case, mode):
    T, H, W, win, sf, at_end = case
    p = make_plan(T=T, H=H, W=W, window=win, sink_frames=sf, sink_at_end=at_end, sparsity=0.6, budget_mode=mode,
                  block=64, head_dim=64)
    perm, inv = p.rf2_plan_perm()
    want = orc.perm_table(T, H, W, *win, sf, bool(at_end))
    assert np.array_equal(perm, want)
    i = p.info
    sb, se = orc.sink_block_range(T * H * W, H * W, 64, sf, bool(at_end))
    assert (i.sink_block_begin, i.sink_block_end) == (sb, se)
    assert (i.k_row, i.k_sel) == orc.budget(i.n_blocks, se - sb, 0.6, mode)
    p.close()


@pytest.mark.parametrize("case", [
    # T, H, W, block, window, sink_frames, text_tokens
    (6, 16, 16, 64, (4, 4, 4), 1, 40), (5, 7, 9, 64, (2, 4, 4), 1, 11), (1, 64, 64, 128, (1, 8, 16), 0, 77),
    (21, 45, 80, 128, (2, 8, 8), 1, 512), (3, 5, 6, 128, (2, 8, 8), 0, 300),
])
def test_text_tokens_tables_match_the_oracle(case):
    T, H, W, b, win, sf, text = case
    p = make_plan(T=T, H=H, W=W, block=b, window=win, sink_frames=sf, text_tokens=text, sparsity=0.7, head_dim=128)
    i = p.info
    N = T * H * W + text
    assert (i.N, i.n_blocks) == (N, orc.n_blocks(N, b))
    sb, se = orc.sink_block_range(N, H * W, b, sf, True, text)
    assert (i.sink_block_begin, i.sink_block_end) == (sb, se)
    assert (i.k_row, i.k_sel) == orc.budget(i.n_blocks, se - sb, 0.7)
    perm, inv = p.rf2_plan_perm()
    want = orc.perm_table(T, H, W, *win, sf, True, text)
    assert np.array_equal(perm, want) and np.array_equal(inv, orc.inverse_table(want))
    p.close()


def test_cdf_mode_reports_capacity_not_a_budget():
    p = make_plan(cdf_threshold=0.8)
    i = p.info
    assert (i.k_row, i.k_sel, i.kept_pairs_per_head, i.achieved_sparsity) == (i.n_blocks, 0, -1, -1.0)
    p.close()


@pytest.mark.parametrize("case", [
    # T, H, W, b_q, b_k, sink_frames, text_tokens, sparsity
    (21, 45, 80, 256, 128, 1, 0, 0.8), (21, 45, 80, 128, 64, 1, 0, 0.8), (6, 16, 16, 64, 128, 1, 0, 0.5),
    (5, 7, 9, 256, 64, 1, 13, 0.6), (1, 40, 36, 128, 64, 0, 0, 0.5), (4, 9, 11, 64, 128, 1, 0, 0.7),
])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_different_q_and_k_blocks_match_the_oracle(case, mode):
    T, H, W, bq, bk, sf, text, s = case
    p = make_plan(T=T, H=H, W=W, block=bq, block_k=bk, sink_frames=sf, text_tokens=text, sparsity=s,
                  budget_mode=mode, head_dim=128)
    i = p.info
    N = T * H * W + text
    Tq, Tk = orc.n_blocks(N, bq), orc.n_blocks(N, bk)
    assert (i.N, i.n_blocks, i.n_blocks_k, i.block_k) == (N, Tq, Tk, bk)
    assert (i.N_pad, i.N_pad_k) == (Tq * bq, Tk * bk)
    assert (i.last_block_valid, i.last_block_valid_k) == (N - (Tq - 1) * bq, N - (Tk - 1) * bk)
    rq = orc.sink_block_range(N, H * W, bq, sf, True, text)
    rk = orc.sink_block_range(N, H * W, bk, sf, True, text)
    assert (i.sink_block_begin, i.sink_block_end) == rq and (i.sink_block_begin_k, i.sink_block_end_k) == rk
    k_row, k_sel = orc.budget(Tq, rq[1] - rq[0], s, mode, Tk, rk[1] - rk[0])
    assert (i.k_row, i.k_sel) == (k_row, k_sel)
    assert i.kept_pairs_per_head == orc.kept_pairs(Tq, rq[1] - rq[0], k_row, Tk)
    assert abs(i.achieved_sparsity - (1 - i.kept_pairs_per_head / (Tq * Tk))) < 1e-12
    assert (i.wt, i.wh, i.ww) == orc.default_window(bq, T > 1)
    p.close()


def test_equal_blocks_report_the_same_k_side():
    p = make_plan()
    i = p.info
    assert (i.block_k, i.n_blocks_k, i.N_pad_k, i.last_block_valid_k) == (64, i.n_blocks, i.N_pad, i.last_block_valid)
    assert (i.sink_block_begin_k, i.sink_block_end_k) == (i.sink_block_begin, i.sink_block_end)
    p.close()


def test_bench_reports_traffic_only_for_the_kernel_source_it_was_measured_on(tmp_path, monkeypatch):
    """bench.py's roofline.traffic comes from a table keyed by the hash of the attention kernel's source;
    a figure measured on another version of the kernel must not be reported."""
    import sys
    sys.path.insert(0, ROOT)
    import bench
    here = bench.attn_source_hash()
    assert len(here) == 16 and int(here, 16) >= 0
    table = tmp_path / "attn_traffic.txt"
    table.write_text(f"# comment\nvideo720p 0000000000000000 9.9e11 stale\nvideo720p {here} 1.5e11 current\nimage {here} 7e8 x\n")
    monkeypatch.setattr(bench, "TRAFFIC_TABLE", str(table))
    assert bench.measured_traffic("video720p") == 1.5e11
    assert bench.measured_traffic("image") == 7e8
    assert bench.measured_traffic("video480p") is None
    table.write_text("video720p 0000000000000000 9.9e11 stale\n")
    assert bench.measured_traffic("video720p") is None
    monkeypatch.setattr(bench, "TRAFFIC_TABLE", str(tmp_path / "missing.txt"))
    assert bench.measured_traffic("video720p") is None
    # the table in the tree has an entry for the source in the tree
    monkeypatch.undo()
    assert bench.measured_traffic("video720p") is not None, "profiles/attn_traffic.txt is stale: re-measure FETCH_SIZE / WRITE_SIZE"
