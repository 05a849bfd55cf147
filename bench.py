#!/usr/bin/env python3
"""Benchmark of the RainFusion2.0 attention layer on one MI355X.

A "step" is one pass of the whole layer -- permute+pool, mask prediction, block-sparse
attention, unpermute -- over one synthetic batch of the headline workload (720p video DiT:
1 x 40 heads x d128, 21x45x80 = 75,600 tokens, block 128, sparsity 0.8, first-frame sink).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu] [--no-dense]
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2512_24086_amd import inputs, rf2  # noqa: E402

METRIC = "ms/layer + effective TFLOPS of block-sparse attn @80% sparsity, 75.6K tokens"
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
# HBM/fabric bytes per launch of the attention kernel come from rocprofv3 --pmc runs (FETCH_SIZE and
# WRITE_SIZE, scaled by a copy kernel of known size).  They are kept in a small table beside the profile
# summaries, one line per measurement: workload, hash of the kernel source it was measured on, bytes.
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "attn_traffic.txt")
ATTN_SOURCE = os.path.join(ROOT, "paper_2512_24086_amd", "csrc", "rf2_attn.hip")


def attn_source_hash() -> str:
    import hashlib
    with open(ATTN_SOURCE, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def measured_traffic(workload: str):
    """Bytes per launch measured for `workload` on exactly the kernel source that is in the tree, else None
    (a figure measured on another version of the kernel says nothing about this one)."""
    try:
        here = attn_source_hash()
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                cols = line.split()
                if len(cols) >= 3 and not line.startswith("#") and cols[0] == workload and cols[1] == here:
                    return float(cols[2])
    except OSError:
        pass
    return None


class PowerSampler:
    """Socket power from the amdgpu hwmon files (microwatts), sampled by a thread every 20 ms; None where
    the files are missing or unreadable.  Samples of the first `skip_s` seconds are dropped (the power
    management needs a moment to settle on a kernel's own level)."""

    def __init__(self, skip_s=0.0):
        import glob
        self.files = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.cap = None
        for f in self.files[:1]:
            try:
                self.cap = int(open(f.replace("power1_input", "power1_cap")).read()) * 1e-6
            except (OSError, ValueError):
                pass
        self.skip_s, self.samples, self._stop, self._thread = skip_s, [], False, None

    def _run(self):
        t0 = time.perf_counter()
        while not self._stop:
            try:
                w = int(open(self.files[0]).read()) * 1e-6
                if time.perf_counter() - t0 >= self.skip_s:
                    self.samples.append(w)
            except (OSError, ValueError):
                return
            time.sleep(0.02)

    def __enter__(self):
        if self.files:
            import threading
            self._thread = threading.Thread(target=self._run, daemon=True)
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        if self._thread:
            self._thread.join()

    def mean(self):
        return round(sum(self.samples) / len(self.samples), 1) if self.samples else None


def power_report(plan, buf):
    """What the chip draws and sustains: the attention kernel looped for ~1.5 s, and a loop of nothing but
    bf16 MFMAs on pseudo-random operands for as long, each with the socket power sampled beside it."""
    call = lambda: plan.rf2_block_sparse_attn_unpermuted(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"],
                                                         buf["blk_cnt"], buf["o"])
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(); call(); b.record(); torch.cuda.synchronize()
    one = max(a.elapsed_time(b), 0.05)
    n_warm, n_timed = max(2, int(500 / one)), max(3, int(1000 / one))
    with PowerSampler(skip_s=0.5) as ps:
        for _ in range(n_warm):
            call()
        torch.cuda.synchronize()
        a.record()
        for _ in range(n_timed):
            call()
        b.record()
        torch.cuda.synchronize()
    attn_ms, attn_w, cap = a.elapsed_time(b) / n_timed, ps.mean(), ps.cap
    with PowerSampler(skip_s=0.5) as ps:
        sustained = rf2.rf2_measure_sustained_mfma(1.5)
    return {"power_cap_w": cap, "attn_steady_ms": round(attn_ms, 4), "attn_power_w": attn_w,
            "mfma_random_operands_sustained_tflops": round(sustained, 1), "mfma_random_operands_power_w": ps.mean()}


def ensure_library():
    if not os.path.exists(rf2.LIB_PATH):
        from paper_2512_24086_amd.build import build
        build(verbose=False)
    rf2.lib()


def time_layer(plan, q, k, v, buf, steps, warmup, fused=True):
    """Times `steps` whole layers (wall clock between device syncs) and each stage (events).
    fused: the inverse permutation happens in the attention kernel's epilogue (3 launches per layer);
    otherwise attention writes the permuted output and rf2_unpermute follows (4 launches)."""
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]

    def one(marks=None):
        if marks: marks[0].record()
        plan.rf2_permute(q, k, v, buf["qp"], buf["kp"], buf["vp"], buf["qbar"], buf["kbar"])
        if marks: marks[1].record()
        plan.rf2_predict_mask(buf["qbar"], buf["kbar"], buf["blk_idx"], buf["blk_cnt"])
        if marks: marks[2].record()
        if fused:
            plan.rf2_block_sparse_attn_unpermuted(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"], buf["blk_cnt"],
                                                  buf["o"])
            if marks: marks[3].record()
        else:
            plan.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"], buf["blk_cnt"], buf["op"])
            if marks: marks[3].record()
            plan.rf2_unpermute(buf["op"], buf["o"])
        if marks: marks[4].record()

    for _ in range(warmup):
        one()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        one(ev[s])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    names = ["permute_pool", "predict_mask", "block_sparse_attn", "unpermute"]
    per_step = {n: sorted(ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(steps)) for i, n in enumerate(names)}
    stages = {n: sum(t) / steps for n, t in per_step.items()}
    spread = {n: {"median": t[steps // 2], "min": t[0]} for n, t in per_step.items()}
    return wall_ms, stages, spread


def time_attn_only(plan, buf, idx, cnt, iters, warmup=1):
    for _ in range(warmup):
        plan.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], idx, cnt, buf["op"])
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        plan.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], idx, cnt, buf["op"])
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


def time_sdpa(q, k, v, iters=5):
    """Library dense attention on the same GPU (context for the dense side of the speedup): every fused
    backend of torch's scaled_dot_product_attention that accepts the problem is timed by name; returns
    (best time in ms, name of that backend, {name: ms or reason})."""
    from torch.nn.attention import SDPBackend, sdpa_kernel
    f = torch.nn.functional.scaled_dot_product_attention
    tried = {}
    for backend in (SDPBackend.FLASH_ATTENTION, SDPBackend.EFFICIENT_ATTENTION):
        try:
            with sdpa_kernel(backend):
                f(q, k, v)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(iters):
                    f(q, k, v)
                b.record()
                torch.cuda.synchronize()
                tried[backend.name] = a.elapsed_time(b) / iters
        except Exception as e:  # noqa: BLE001 -- report, never fail the bench on the context number
            tried[backend.name] = f"unavailable: {type(e).__name__}"
    timed = {n: t for n, t in tried.items() if isinstance(t, float)}
    if not timed:
        return None, None, tried
    best = min(timed, key=timed.get)
    return timed[best], best, tried


def mask_diagnostics(orc, plan, buf, head, Qp, Kp, S_hat, M):
    """Near-tie rows of one head (selection-boundary gap <= 1e-3 in the oracle's scores: the rows where
    several masks are correct), how many of them the GPU resolved differently, and the share of the dense
    attention mass the mask keeps on 256 seeded query rows."""
    import numpy as np
    i, c = plan.info, plan.cfg
    Tq, Tk = i.n_blocks, i.n_blocks_k
    idx, cnt = buf["blk_idx"][0, head].cpu().numpy(), buf["blk_cnt"][0, head].cpu().numpy()
    M_gpu = np.zeros((Tq, Tk), dtype=bool)
    for r in range(Tq):
        if cnt[r] == Tk:
            M_gpu[r] = True
        else:
            M_gpu[r, idx[r, :cnt[r]]] = True
    out = {"head": head}
    if c.select_mode == rf2.RF2_SELECT_TOPN:
        gap = orc.selection_gap(S_hat, i.k_sel, i.sink_block_begin, i.sink_block_end,
                                (i.sink_block_begin_k, i.sink_block_end_k))
        near = gap <= 1e-3
        out.update({"near_tie_rows": int(near.sum()), "rows": int(np.isfinite(gap).sum()),
                    "near_tie_rows_resolved_differently": int((M_gpu[near] != M[near]).any(axis=1).sum()),
                    "other_rows_differing": int((M_gpu[~near] != M[~near]).any(axis=1).sum())})
    rows = np.sort(np.random.default_rng(0).choice(int(i.N), min(256, int(i.N)), replace=False))
    out["dense_attention_mass_kept"] = round(orc.attention_mass_recall(Qp, Kp, M_gpu, c.block, i.block_k, rows), 4)
    out["kept_density"] = round(float(M_gpu[rows // c.block].mean()), 4)
    return out


def cpu_baseline(wl, plan, q, k, v, buf, dense_flops):
    """The fp64 oracle, untuned, on a bounded sample: all stages for ONE head up to the mask, attention
    for the Q blocks of that head; extrapolated to the whole layer by head count and kept pairs."""
    from oracle import rf2_oracle as orc
    from threadpoolctl import threadpool_info
    i, c = plan.info, plan.cfg
    head = 0
    Q, K, V = (orc.bf16_bits_to_f64(inputs.bf16_bits(x[0, head])) for x in (q, k, v))
    t0 = time.perf_counter()
    perm = orc.perm_table(c.T, c.H, c.W, i.wt, i.wh, i.ww, c.sink_frames, bool(c.sink_at_end), c.text_tokens)
    Qp, Kp, Vp = orc.permute(Q, perm), orc.permute(K, perm), orc.permute(V, perm)
    S_hat = orc.block_scores(orc.pool_blocks(Qp, c.block), orc.pool_blocks(Kp, i.block_k))
    sink_k = (i.sink_block_begin_k, i.sink_block_end_k)
    if c.select_mode == rf2.RF2_SELECT_CDF:
        M, _ = orc.select_blocks_cdf(S_hat, float(c.cdf_threshold), c.head_dim, i.sink_block_begin, i.sink_block_end,
                                     sink_k)
    else:
        M = orc.select_blocks(S_hat, i.k_sel, i.sink_block_begin, i.sink_block_end, sink_k)
    t_pre = time.perf_counter() - t0
    diag = mask_diagnostics(orc, plan, buf, head, Qp, Kp, S_hat, M)
    Tb = i.n_blocks
    sample = list(range(Tb))                           # every Q block of this one head: ~10 s of oracle time
    t0 = time.perf_counter()
    Op = orc.block_sparse_attention(Qp, Kp, Vp, M, c.block, q_blocks=sample, bk=i.block_k)
    t_attn = time.perf_counter() - t0
    pairs = int(sum(M[r].sum() for r in sample))
    t_unp0 = time.perf_counter()
    orc.unpermute(Op, perm)
    t_unp = time.perf_counter() - t_unp0
    per_head = t_pre + t_unp + t_attn * (int(M.sum()) / pairs)
    layer_s = per_head * c.batch * c.heads
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": dense_flops / layer_s / 1e12, "unit": "TFLOP/s dense-equivalent (extrapolated)",
            "cores": threads, "kind": "oracle", "ms_per_layer_extrapolated": layer_s * 1e3, "mask": diag,
            "sample": f"head {head}: permute+pool+scores+selection in full ({t_pre:.2f} s), attention on "
                      f"{len(sample)} of {Tb} Q blocks = {pairs} block pairs ({t_attn:.2f} s), scaled by "
                      f"kept pairs and by {c.batch * c.heads} heads"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="video720p", choices=list(inputs.WORKLOADS))
    ap.add_argument("--sparsity", type=float, default=None)
    ap.add_argument("--text-tokens", type=int, default=0,
                    help="append this many text tokens (always-dense rows and columns) to the video tokens")
    ap.add_argument("--head-dim", type=int, default=None, choices=(64, 128), help="override the workload's head_dim")
    ap.add_argument("--block", type=int, default=None, choices=(64, 128, 256),
                    help="override the workload's block size (b_q; also b_k unless --block-k is given)")
    ap.add_argument("--block-k", type=int, default=0, choices=(0, 64, 128), help="K/V block size b_k if different")
    ap.add_argument("--cdf", type=float, default=None,
                    help="cumulative-mass block selection with this threshold instead of top-n (row lengths vary)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense-attention baselines")
    ap.add_argument("--no-power", action="store_true", help="skip the power / sustained-MFMA measurement (~3 s)")
    ap.add_argument("--unfused", action="store_true",
                    help="time rf2_block_sparse_attn + rf2_unpermute instead of the fused entry point")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a single-GPU kernel path; run with --gpus 1 "
              "(heads shard across GPUs with no communication, nothing multi-GPU is implemented)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    ensure_library()
    torch.cuda.set_device(0)
    wl = inputs.WORKLOADS[args.workload]
    if args.text_tokens:
        wl = dataclasses.replace(wl, text_tokens=args.text_tokens)
    if args.head_dim or args.block:
        wl = dataclasses.replace(wl, head_dim=args.head_dim or wl.head_dim, block=args.block or wl.block)
    s = wl.sparsity if args.sparsity is None else args.sparsity
    plan = rf2.Plan(batch=wl.batch, heads=wl.heads, head_dim=wl.head_dim, T=wl.T, H=wl.H, W=wl.W, block=wl.block,
                    sparsity=s, sink_frames=wl.sink_frames, text_tokens=wl.text_tokens, cdf_threshold=args.cdf,
                    block_k=args.block_k)
    i = plan.info
    q, k, v = inputs.make_qkv(wl, device="cuda")
    buf = plan.alloc("cuda")
    torch.cuda.synchronize()

    wall_ms, stages, spread = time_layer(plan, q, k, v, buf, args.steps, args.warmup, fused=not args.unfused)
    mfma_peak, copy_peak = rf2.rf2_measure_peaks()        # ceilings measured on this machine, for context
    bh = wl.batch * wl.heads
    dense_flops = 4.0 * wl.N * wl.N * wl.head_dim * bh
    kept_pairs = i.kept_pairs_per_head * bh
    if args.cdf is not None:            # data dependent: count what the mask kernel kept
        kept_pairs = int(buf["blk_cnt"].sum().item())
    kept_flops = 4.0 * wl.block * i.block_k * wl.head_dim * kept_pairs
    attn_ms = stages["block_sparse_attn"]
    itemsize = 2
    tensor_bytes = bh * wl.N * wl.head_dim * itemsize
    # permute + pool: reads q, k, v; writes the padded permuted copies and the fp32 block means
    permute_bytes = (3 * tensor_bytes + bh * wl.head_dim * itemsize * (i.N_pad + 2 * i.N_pad_k)
                     + bh * wl.head_dim * 4 * (i.n_blocks + i.n_blocks_k))
    gbps = {"permute_pool": permute_bytes / (stages["permute_pool"] * 1e-3) / 1e9}
    if args.unfused:
        gbps["unpermute"] = (2 * tensor_bytes) / (stages["unpermute"] * 1e-3) / 1e9
    else:
        stages["unpermute"] = 0.0          # done by the attention kernel's epilogue
    out = {
        "metric": METRIC, "value": dense_flops / (wall_ms * 1e-3) / 1e12,
        "unit": "TFLOP/s dense-equivalent (4*N^2*d*heads per layer / whole-layer time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: B{wl.batch} x {wl.heads} heads x d{wl.head_dim}, grid {wl.T}x{wl.H}x{wl.W}"
                               f" = {wl.T * wl.H * wl.W} tokens"
                               + (f" + {wl.text_tokens} text tokens" if wl.text_tokens else "")
                               + f", block {wl.block}" + (f" (K/V blocks {i.block_k})" if i.block_k != wl.block else "")
                               + f", sparsity {s}, sink_frames {wl.sink_frames}",
                   "selection": "top-n (eq. 8)" if args.cdf is None else f"cumulative mass >= {args.cdf}",
                   "n_blocks": i.n_blocks, "n_blocks_k": i.n_blocks_k, "k_row": i.k_row,
                   "kept_pairs_per_head": kept_pairs / bh,
                   "achieved_sparsity": round(1.0 - kept_pairs / bh / (i.n_blocks * i.n_blocks_k), 4),
                   "inverse_permutation": "rf2_unpermute" if args.unfused else "fused into the attention epilogue"},
        "stages_ms": {n: round(t, 4) for n, t in stages.items()},
        "stages_ms_median_min": {n: [round(v["median"], 4), round(v["min"], 4)] for n, v in spread.items()
                                 if n != "unpermute" or args.unfused},
        "stages_gbps": {n: round(g, 1) for n, g in gbps.items()},
        "measured_peaks": {"mfma_bf16_loop_tflops": round(mfma_peak, 1), "copy_kernel_gbps": round(copy_peak, 1),
                           "attn_frac_of_mfma_loop": round(kept_flops / (attn_ms * 1e-3) / 1e12 / mfma_peak, 4),
                           "permute_pool_frac_of_copy": round(gbps["permute_pool"] / copy_peak, 4)},
        "attn": {"ms": round(attn_ms, 4), "kept_tflops": round(kept_flops / (attn_ms * 1e-3) / 1e12, 1),
                 "dense_equiv_tflops": round(dense_flops / (attn_ms * 1e-3) / 1e12, 1)},
        "roofline": {"bound": "mfma", "kernel": "block_sparse_attn_kernel",
                     "achieved": kept_flops / (attn_ms * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": kept_flops / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "traffic": (measured_traffic(wl.name)
                                 if args.sparsity is None and not wl.text_tokens and args.cdf is None
                                 and not args.head_dim and not args.block and not args.block_k else None)},
    }
    if not args.no_power:
        pw = power_report(plan, buf)
        steady_tflops = kept_flops / (pw["attn_steady_ms"] * 1e-3) / 1e12
        pw["attn_steady_kept_tflops"] = round(steady_tflops, 1)
        pw["attn_frac_of_sustained_mfma"] = round(steady_tflops / pw["mfma_random_operands_sustained_tflops"], 4)
        out["power"] = pw
    if not args.no_dense:
        cnt_dense = torch.full_like(buf["blk_cnt"], i.n_blocks_k)
        dense_ms = time_attn_only(plan, buf, buf["blk_idx"], cnt_dense, iters=5)
        sdpa_ms, sdpa_backend, sdpa_all = time_sdpa(q, k, v)
        best = min(dense_ms, sdpa_ms) if sdpa_ms is not None else dense_ms
        out["attn"].update({"dense_same_kernel_ms": round(dense_ms, 3),
                            "dense_torch_sdpa_ms": round(sdpa_ms, 3) if sdpa_ms is not None else None,
                            "dense_torch_sdpa_backend": sdpa_backend,
                            "dense_torch_sdpa_backends_tried": {n: (round(t, 3) if isinstance(t, float) else t)
                                                                for n, t in sdpa_all.items()},
                            "speedup_vs_fastest_dense": round(best / attn_ms, 3)})
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl, plan, q, k, v, buf, dense_flops)
        out["near_tie_rows"] = out["cpu_baseline"]["mask"].get("near_tie_rows")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
