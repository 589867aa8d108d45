"""The read-rate measurement aid: sizes it reports, and the buffers it refuses on the host."""
from __future__ import annotations

import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_read_sweep_reports_bytes_and_refuses_foreign_memory():
    import torch
    from paper_2501_08547_amd import binding as B
    dev = "cuda:0"
    ctx = B.Context(torch.zeros(2, dtype=torch.int64, device=dev), torch.zeros(1, dtype=torch.int32, device=dev))
    try:
        buf = torch.ones(8 << 18, dtype=torch.float32, device=dev)             # 8 MiB
        nbytes, ms = ctx.measure_read_rate(buf, reps=3, blocks=64)
        # 64 blocks x 256 lanes x 4 loads of 16 bytes = 1 MiB per turn: 8 MiB = 8 turns, all of them whole
        assert nbytes == 3 * float(8 << 20)
        assert ms > 0.0
        L = B.lib()
        nb, t = C.c_double(0.0), C.c_float(0.0)
        host = np.zeros(8 << 18, dtype=np.float32)
        assert L.omg_measure_read_rate(ctx.handle, host.ctypes.data, host.nbytes, 1, 64, C.byref(nb), C.byref(t)) == B.OMG_EINVAL
        # more bytes than the allocation that holds the buffer
        big = torch.ones(64 << 18, dtype=torch.float32, device=dev)            # a 64 MiB block of its own
        assert L.omg_measure_read_rate(ctx.handle, big.data_ptr(), (64 << 20) + (1 << 30), 1, 64,
                                       C.byref(nb), C.byref(t)) == B.OMG_EINVAL
        # fewer pieces than one turn of the grid needs
        assert L.omg_measure_read_rate(ctx.handle, buf.data_ptr(), 8 << 20, 1, 1024, C.byref(nb), C.byref(t)) == B.OMG_EINVAL
        # the refused calls left no error behind
        nbytes2, _ = ctx.measure_read_rate(buf, reps=1, blocks=64)
        assert nbytes2 == float(8 << 20)
    finally:
        ctx.close()
