"""The selection entry point that owns its scratch (toma_select_static): called through the C ABI,
its picks, values and leads must be those of toma_select, bit for bit, on two calls in a row, the
second on a smaller input (the shared static buffer then still holds the first call's similarities);
shapes beyond the buffer are refused on the host."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2509_10918_amd import binding as tb
from paper_2509_10918_amd import synth

import toma_gpu as tg

W = synth.WORKLOADS


def _both(w):
    inp = synth.make_inputs(w)
    dv = tg.Device(w, inp, 1)
    ref_idx = dv.select().copy()
    ref_gain, ref_gap = dv.gain.cpu().numpy().copy(), dv.gap.cpu().numpy().copy()
    idx = torch.full_like(dv.idx, -1)
    gain, gap = torch.full_like(dv.gain, np.nan), torch.full_like(dv.gap, np.nan)
    L = tb.lib()
    rc = L.toma_select_static(ctypes.addressof(dv.desc), dv.X.data_ptr(), idx.data_ptr(), gain.data_ptr(),
                              gap.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0, tb.status_string(rc)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), ref_idx)
    assert np.array_equal(gain.cpu().numpy(), ref_gain)
    assert np.array_equal(gap.cpu().numpy(), ref_gap)
    return ref_idx


@pytest.mark.gpu
def test_select_static_matches_select_twice_then_smaller(oracle):
    big = synth.scaled(W["sdxl1"], name="static_big", B=2, H=48, W=64, C=128, heads=2, index=23)
    small = synth.scaled(W["sdxl2"], name="static_small", B=1, H=16, W=24, C=64, heads=1, index=24)
    print(f"[static] {big.B}x{big.P} regions of {big.n_loc}, then {small.B}x{small.P} regions of {small.n_loc}", flush=True)
    idx_big = _both(big)
    idx_small = _both(small)
    _both(big)
    # and the picks are the oracle's
    for w, idx in ((big, idx_big), (small, idx_small)):
        X = np.asarray(synth.make_inputs(w)["X"], np.float64)
        bad, _, _ = tg.compare_picks(oracle, w, X, idx)
        assert not bad


def test_select_static_refuses_what_does_not_fit():
    """Host-side checks only: nothing is launched."""
    L = tb.lib()
    x = 1 << 20
    hires = tb.make_desc(2, 128, 128, 640, 16, 16, 128, 1, 0.1, "bf16")   # 32 MiB of similarities
    assert L.toma_select_static(ctypes.addressof(hires), x, x, None, None, None) == 4
    ok = tb.make_desc(2, 64, 64, 640, 16, 16, 128, 1, 0.1, "bf16")
    assert L.toma_select_static(ctypes.addressof(ok), None, x, None, None, None) == 1
    assert L.toma_select_static(ctypes.addressof(ok), x + 2, x, None, None, None) == 3
    assert L.toma_select_static(None, x, x, None, None, None) == 1
