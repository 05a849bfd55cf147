"""The allocation-free XCD probe (rf2_probe_xcd_mapping_static) against the allocating one, through the C-ABI.

Two calls in a row share the library's static device array; the second launches fewer workgroups, so the
array still holds entries of the first call beyond the ones the second call reads."""
import ctypes as C

import pytest
import torch

from paper_2512_24086_amd import rf2

pytestmark = pytest.mark.gpu

MAX_WG = 8192   # RF2_XCD_PROBE_MAX_WORKGROUPS in include/rf2.h


def _allocating_probe(lib):
    agree, total, first = C.c_int32(0), C.c_int32(0), C.c_int32(-1)
    assert lib.rf2_probe_xcd_mapping(C.byref(agree), C.byref(total), C.byref(first), None) == rf2.RF2_OK
    return agree.value, total.value, first.value


def _static_probe(lib, n, result, stream):
    rc = lib.rf2_probe_xcd_mapping_static(C.c_int32(n), C.c_void_p(result.data_ptr()), C.c_void_p(stream))
    assert rc == rf2.RF2_OK, rf2.lib().rf2_strerror(rc)


def test_static_probe_equals_the_allocating_probe_on_two_calls_in_a_row():
    lib = rf2.lib()
    ref_agree, ref_total, ref_first = _allocating_probe(lib)
    assert ref_total == MAX_WG and 0 <= ref_first < 8
    stream = torch.cuda.current_stream().cuda_stream
    result = torch.full((2,), -7, dtype=torch.int32, device="cuda")

    # first call: as many workgroups as the allocating probe launches -> the same count, exactly
    _static_probe(lib, MAX_WG, result, stream)
    torch.cuda.synchronize()
    agree, first = result.tolist()
    print(f"static probe, {MAX_WG} workgroups: {agree} agree (allocating probe: {ref_agree} of {ref_total}), "
          f"workgroup 0 on XCD {first}")
    assert agree == ref_agree
    assert 0 <= first < 8          # which XCD a launch starts on is not fixed: only its range is checked

    # second call, smaller: entries 1000.. of the array still hold the first call's values.  The
    # allocating probe has a fixed size; what it says about every residue class (all of its
    # workgroups agree, or the classes are not on 8 different XCDs and none does) carries over.
    n_small = 1000
    result.fill_(-7)
    _static_probe(lib, n_small, result, stream)
    torch.cuda.synchronize()
    agree_small, first_small = result.tolist()
    assert ref_agree in (0, ref_total)
    assert agree_small == (n_small if ref_agree == ref_total else 0)
    assert 0 <= first_small < 8

    # and the allocating probe still answers the same afterwards
    assert _allocating_probe(lib)[:2] == (ref_agree, ref_total)


def test_static_probe_can_be_captured_and_replayed():
    # a hipMalloc, a host copy or a synchronisation inside the call would make the capture fail
    lib = rf2.lib()
    ref_agree, ref_total, _ = _allocating_probe(lib)
    result = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    side = torch.zeros(1 << 20, device="cuda")
    _static_probe(lib, 512, result, torch.cuda.current_stream().cuda_stream)   # first call on the device: symbol lookup
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _static_probe(lib, 4096, result, torch.cuda.current_stream().cuda_stream)
    for replay in range(3):
        result.fill_(-7)
        side.add_(1.0)                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        agree, first = result.tolist()
        assert agree == (4096 if ref_agree == ref_total else 0), (replay, agree)
        assert 0 <= first < 8
