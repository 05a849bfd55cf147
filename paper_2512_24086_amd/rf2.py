"""Thin ctypes binding of librf2.so: same names as the C ABI, argument marshalling only.

PyTorch supplies device memory and streams; every step of the layer runs in the HIP
kernels of the library.  There is no fallback: if librf2.so is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "librf2.so")

RF2_OK = 0
RF2_ERR_INVALID_ARG, RF2_ERR_UNSUPPORTED, RF2_ERR_ALLOC, RF2_ERR_HIP, RF2_ERR_TOO_LARGE = -1, -2, -3, -4, -5
RF2_BUDGET_GLOBAL, RF2_BUDGET_ROW_INCL_SINK, RF2_BUDGET_ROW_PLUS_SINK = 0, 1, 2
RF2_LAYOUT_BHND, RF2_LAYOUT_BNHD = 0, 1
RF2_SELECT_TOPN, RF2_SELECT_CDF = 0, 1


class rf2_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "heads", "head_dim", "T", "H", "W", "wt", "wh", "ww",
                                         "block", "sink_frames", "sink_at_end")] + \
               [("sparsity", C.c_float), ("budget_mode", C.c_int32), ("qkv_layout", C.c_int32), ("text_tokens", C.c_int32),
                ("select_mode", C.c_int32), ("cdf_threshold", C.c_float), ("block_k", C.c_int32)]


class rf2_info(C.Structure):
    _fields_ = [("N", C.c_int64), ("N_pad", C.c_int64), ("n_blocks", C.c_int32), ("last_block_valid", C.c_int32),
                ("sink_block_begin", C.c_int32), ("sink_block_end", C.c_int32), ("k_row", C.c_int32),
                ("k_sel", C.c_int32), ("wt", C.c_int32), ("wh", C.c_int32), ("ww", C.c_int32),
                ("kept_pairs_per_head", C.c_int64), ("achieved_sparsity", C.c_double),
                ("workspace_bytes", C.c_int64), ("block_k", C.c_int32), ("n_blocks_k", C.c_int32),
                ("last_block_valid_k", C.c_int32), ("sink_block_begin_k", C.c_int32), ("sink_block_end_k", C.c_int32),
                ("N_pad_k", C.c_int64)]


# symbol -> (restype, argtypes); also the list of exports the tests check
SIGNATURES = {
    "rf2_plan_create": (C.c_int, [C.POINTER(rf2_config), C.POINTER(C.c_void_p)]),
    "rf2_plan_destroy": (C.c_int, [C.c_void_p]),
    "rf2_plan_info": (C.c_int, [C.c_void_p, C.POINTER(rf2_info)]),
    "rf2_plan_perm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "rf2_permute": (C.c_int, [C.c_void_p] * 10),
    "rf2_predict_mask": (C.c_int, [C.c_void_p] * 9),
    "rf2_block_sparse_attn": (C.c_int, [C.c_void_p] * 9),
    "rf2_block_sparse_attn_unpermuted": (C.c_int, [C.c_void_p] * 9),
    "rf2_unpermute": (C.c_int, [C.c_void_p] * 4),
    "rf2_measure_peaks": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]),
    "rf2_measure_sustained_mfma": (C.c_int, [C.c_double, C.POINTER(C.c_double), C.c_void_p]),
    "rf2_probe_xcd_mapping": (C.c_int, [C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_void_p]),
    "rf2_probe_xcd_mapping_static": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p]),
    "rf2_strerror": (C.c_char_p, [C.c_int]),
    "rf2_version": (C.c_int, []),
}

_lib = None


def lib() -> C.CDLL:
    """Loads librf2.so (built beforehand by paper_2512_24086_amd.build); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2512_24086_amd.build` "
                               "(there is no fallback implementation)")
        _lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(_lib, name)
            fn.restype, fn.argtypes = res, args
    return _lib


class Rf2Error(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().rf2_strerror(code).decode()} ({code})")


def _check(code: int, where: str) -> None:
    if code != RF2_OK:
        raise Rf2Error(code, where)


def _ptr(t) -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    assert t.is_contiguous(), "tensors handed to librf2 must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def rf2_measure_peaks(stream=None):
    """(bf16 MFMA-loop TFLOP/s, copy-kernel GB/s) measured on the current device."""
    mfma, copy = C.c_double(0.0), C.c_double(0.0)
    _check(lib().rf2_measure_peaks(C.byref(mfma), C.byref(copy), _stream(stream)), "rf2_measure_peaks")
    return mfma.value, copy.value


def rf2_measure_sustained_mfma(seconds, stream=None):
    """bf16 MFMA TFLOP/s sustained for `seconds` on pseudo-random operands (the power-limited ceiling)."""
    out = C.c_double(0.0)
    _check(lib().rf2_measure_sustained_mfma(C.c_double(seconds), C.byref(out), _stream(stream)),
           "rf2_measure_sustained_mfma")
    return out.value


def rf2_probe_xcd_mapping(stream=None):
    """(workgroups on the XCD of their residue class g % 8, workgroups launched, XCD of workgroup 0)."""
    agree, total, first = C.c_int32(0), C.c_int32(0), C.c_int32(-1)
    _check(lib().rf2_probe_xcd_mapping(C.byref(agree), C.byref(total), C.byref(first), _stream(stream)),
           "rf2_probe_xcd_mapping")
    return agree.value, total.value, first.value


def rf2_probe_xcd_mapping_static(n_launch, result, stream=None):
    """Allocation-free probe: leaves (agreeing workgroups, XCD of workgroup 0) in `result` (device int32[2])."""
    _check(lib().rf2_probe_xcd_mapping_static(C.c_int32(n_launch), _ptr(result), _stream(stream)),
           "rf2_probe_xcd_mapping_static")


class Plan:
    """Owner of an rf2_plan*; methods carry the names of the C entry points."""

    def __init__(self, *, batch, heads, head_dim, T, H, W, block, sparsity, sink_frames=0, sink_at_end=1,
                 window=(0, 0, 0), budget_mode=RF2_BUDGET_GLOBAL, qkv_layout=RF2_LAYOUT_BHND, text_tokens=0,
                 cdf_threshold=None, block_k=0):
        self.cfg = rf2_config(batch, heads, head_dim, T, H, W, window[0], window[1], window[2], block,
                              sink_frames, int(sink_at_end), float(sparsity), budget_mode, qkv_layout, text_tokens,
                              RF2_SELECT_TOPN if cdf_threshold is None else RF2_SELECT_CDF,
                              0.0 if cdf_threshold is None else float(cdf_threshold), block_k)
        self._h = C.c_void_p(0)
        _check(lib().rf2_plan_create(C.byref(self.cfg), C.byref(self._h)), "rf2_plan_create")
        self.info = rf2_info()
        _check(lib().rf2_plan_info(self._h, C.byref(self.info)), "rf2_plan_info")

    def close(self):
        if self._h:
            lib().rf2_plan_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- host tables -------------------------------------------------------------------
    def rf2_plan_perm(self):
        import numpy as np
        perm = np.empty(self.info.N, dtype=np.int32)
        inv = np.empty(self.info.N, dtype=np.int32)
        _check(lib().rf2_plan_perm(self._h, perm.ctypes.data, inv.ctypes.data), "rf2_plan_perm")
        return perm, inv

    # -- buffers (allocation only) -----------------------------------------------------------
    def alloc(self, device="cuda", dense_mask=False, scores=False, lse=False):
        c, i = self.cfg, self.info
        bh = (c.batch, c.heads)
        bf = dict(dtype=torch.bfloat16, device=device)
        buf = dict(
            qp=torch.empty(*bh, i.N_pad, c.head_dim, **bf),
            kp=torch.empty(*bh, i.n_blocks_k, i.block_k // 64, c.head_dim // 8, 64, 8, **bf),
            vp=torch.empty(*bh, i.n_blocks_k, i.block_k // 64, 8, c.head_dim, 8, **bf),
            qbar=torch.empty(*bh, i.n_blocks, c.head_dim, dtype=torch.float32, device=device),
            kbar=torch.empty(*bh, i.n_blocks_k, c.head_dim, dtype=torch.float32, device=device),
            blk_idx=torch.empty(*bh, i.n_blocks, i.k_row, dtype=torch.int32, device=device),
            blk_cnt=torch.empty(*bh, i.n_blocks, dtype=torch.int32, device=device),
            op=torch.empty(*bh, i.N_pad, c.head_dim, **bf),
            o=(torch.empty(c.batch, i.N, c.heads, c.head_dim, **bf) if c.qkv_layout == RF2_LAYOUT_BNHD
               else torch.empty(*bh, i.N, c.head_dim, **bf)))
        if dense_mask:
            buf["mask_dense"] = torch.empty(*bh, i.n_blocks, i.n_blocks_k, dtype=torch.uint8, device=device)
        if scores:
            buf["scores"] = torch.empty(*bh, i.n_blocks, i.n_blocks_k, dtype=torch.float32, device=device)
        if lse:
            buf["lse"] = torch.empty(*bh, i.N_pad, dtype=torch.float32, device=device)
        return buf

    # -- the four calls --------------------------------------------------------------------
    def rf2_permute(self, q, k, v, qp, kp, vp, qbar=None, kbar=None, stream=None):
        _check(lib().rf2_permute(self._h, _ptr(q), _ptr(k), _ptr(v), _ptr(qp), _ptr(kp), _ptr(vp), _ptr(qbar),
                                 _ptr(kbar), _stream(stream)), "rf2_permute")

    def rf2_predict_mask(self, qbar, kbar, blk_idx, blk_cnt, mask_dense=None, scores=None, workspace=None,
                         stream=None):
        _check(lib().rf2_predict_mask(self._h, _ptr(qbar), _ptr(kbar), _ptr(blk_idx), _ptr(blk_cnt),
                                      _ptr(mask_dense), _ptr(scores), _ptr(workspace), _stream(stream)),
               "rf2_predict_mask")

    def rf2_block_sparse_attn(self, qp, kp, vp, blk_idx, blk_cnt, op, lse=None, stream=None):
        _check(lib().rf2_block_sparse_attn(self._h, _ptr(qp), _ptr(kp), _ptr(vp), _ptr(blk_idx), _ptr(blk_cnt),
                                           _ptr(op), _ptr(lse), _stream(stream)), "rf2_block_sparse_attn")

    def rf2_block_sparse_attn_unpermuted(self, qp, kp, vp, blk_idx, blk_cnt, o, lse=None, stream=None):
        _check(lib().rf2_block_sparse_attn_unpermuted(self._h, _ptr(qp), _ptr(kp), _ptr(vp), _ptr(blk_idx),
                                                      _ptr(blk_cnt), _ptr(o), _ptr(lse), _stream(stream)),
               "rf2_block_sparse_attn_unpermuted")

    def rf2_unpermute(self, op, o, stream=None):
        _check(lib().rf2_unpermute(self._h, _ptr(op), _ptr(o), _stream(stream)), "rf2_unpermute")

    def layer_fused(self, q, k, v, buf, stream=None):
        """The whole layer with the inverse permutation fused into the attention epilogue; returns buf['o']."""
        self.rf2_permute(q, k, v, buf["qp"], buf["kp"], buf["vp"], buf["qbar"], buf["kbar"], stream)
        self.rf2_predict_mask(buf["qbar"], buf["kbar"], buf["blk_idx"], buf["blk_cnt"], buf.get("mask_dense"),
                              buf.get("scores"), None, stream)
        self.rf2_block_sparse_attn_unpermuted(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"], buf["blk_cnt"],
                                              buf["o"], None, stream)
        return buf["o"]

    def layer(self, q, k, v, buf, stream=None):
        """The whole layer, in order; returns buf['o']."""
        self.rf2_permute(q, k, v, buf["qp"], buf["kp"], buf["vp"], buf["qbar"], buf["kbar"], stream)
        self.rf2_predict_mask(buf["qbar"], buf["kbar"], buf["blk_idx"], buf["blk_cnt"], buf.get("mask_dense"),
                              buf.get("scores"), None, stream)
        self.rf2_block_sparse_attn(buf["qp"], buf["kp"], buf["vp"], buf["blk_idx"], buf["blk_cnt"], buf["op"],
                                   buf.get("lse"), stream)
        self.rf2_unpermute(buf["op"], buf["o"], stream)
        return buf["o"]
