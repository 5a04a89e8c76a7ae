"""The calibration probes: argument handling and plausible rates (the bare matrix-core loop
cannot exceed the published peak and a healthy part sustains well over a third of it; a
streaming read of 256 MiB lands between 2 and 8 TB/s)."""
import ctypes

import pytest
import torch

from paper_2512_12949_amd import binding as ff

pytestmark = pytest.mark.gpu


def test_probe_rates_are_plausible():
    scratch = torch.zeros(16384, dtype=torch.uint8, device="cuda")
    for dt in (ff.DT_BF16, ff.DT_F16):
        rate = ff.ffuse_calibrate(ff.CAL_MFMA, dt, None, 4096, scratch)
        assert 0.35 * 2.5166e15 < rate <= 1.02 * 2.5166e15, rate
    # on all-zero operands the loop runs at what the issue logic allows: close to the published peak, and never
    # slower than on data that toggles the multipliers
    idle = max(ff.ffuse_calibrate(ff.CAL_MFMA_IDLE, ff.DT_BF16, None, 16384, scratch) for _ in range(3))
    busy = max(ff.ffuse_calibrate(ff.CAL_MFMA, ff.DT_BF16, None, 16384, scratch) for _ in range(3))
    assert 0.7 * 2.5166e15 < idle <= 1.02 * 2.5166e15 and idle >= 0.95 * busy, (idle, busy)
    buf = torch.ones(1 << 26, dtype=torch.float32, device="cuda")
    rate = ff.ffuse_calibrate(ff.CAL_READ, ff.DT_BF16, buf, 4, scratch)
    assert 2.0e12 < rate < 8.0e12, rate
    assert bool((scratch == 0).all())            # the probes write nothing in practice
    # a ragged size (not a multiple of the per-step span) is read to its last 16 bytes without touching what follows
    rate = ff.ffuse_calibrate(ff.CAL_READ, ff.DT_BF16, buf[: (1 << 20) + 12], 2, scratch)
    assert rate > 0


def test_probe_argument_errors():
    L = ff.lib()
    scratch = torch.zeros(16384, dtype=torch.uint8, device="cuda")
    buf = torch.ones(1 << 16, dtype=torch.float32, device="cuda")
    out = ctypes.c_double(0.0)
    sp, bp = scratch.data_ptr(), buf.data_ptr()
    assert L.ffuse_calibrate(ff.CAL_MFMA, ff.DT_BF16, None, 0, 16, sp, None, None) == -1
    assert L.ffuse_calibrate(ff.CAL_MFMA, ff.DT_BF16, None, 0, 16, None, ctypes.byref(out), None) == -1
    assert L.ffuse_calibrate(ff.CAL_MFMA, ff.DT_F32, None, 0, 16, sp, ctypes.byref(out), None) == -4
    assert L.ffuse_calibrate(7, ff.DT_BF16, None, 0, 16, sp, ctypes.byref(out), None) == -4
    assert L.ffuse_calibrate(ff.CAL_MFMA, ff.DT_BF16, None, 0, 0, sp, ctypes.byref(out), None) == -2
    assert L.ffuse_calibrate(ff.CAL_READ, ff.DT_BF16, None, 1 << 16, 1, sp, ctypes.byref(out), None) == -1
    assert L.ffuse_calibrate(ff.CAL_READ, ff.DT_BF16, bp + 4, 1 << 16, 1, sp, ctypes.byref(out), None) == -3
    assert L.ffuse_calibrate(ff.CAL_READ, ff.DT_BF16, bp, (1 << 16) + 8, 1, sp, ctypes.byref(out), None) == -2
    torch.cuda.synchronize()
