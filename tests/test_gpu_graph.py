"""A fused call can be captured into a HIP graph and replayed: every launch of the path is a
kernel launch on the caller's stream (no memset nodes, no synchronisation, no allocation),
and the kernels leave flags and counters clean for the next replay.  Replays are interleaved
with eager work and checked against the eager result every time."""
import numpy as np
import pytest
import torch

from paper_2512_12949_amd import binding as ff
from paper_2512_12949_amd import inputs
from paper_2512_12949_amd.inputs import ACT_GELU_TANH, ACT_SILU

import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,gated,plan", [
    ((64, 264, 1304, 520), True, None),                                                    # two-phase, partial planes + finalize
    ((300, 136, 840, 264), False, ("two", dict(bm=128, splits=1, raster=2))),             # two-phase, direct output
    ((300, 136, 840, 264), False, ("reduce", dict(bm=128, bh=64))),                       # atomics + finalize
    ((700, 200, 520, 264), False, ("exchange", dict(producers=16, ring=32))),             # ring + flags
])
def test_fused_call_replays_from_a_graph(shape, gated, plan):
    M, K, N1, N2 = shape
    act = ACT_SILU if gated else ACT_GELU_TANH
    w = inputs.custom("graph", M, K, N1, N2, dtype="bf16", act=act, gated=gated, cfg_id=910)
    host = inputs.make(w)
    dev = {k: gu.to_device(v, "bf16") for k, v in host.items()}
    ref = gu.oracle_rows(w, host)
    p = None
    if plan is not None:
        kind, kw = plan
        if kind == "two":
            p = ff.make_plan(ff.FAMILY_TWOPHASE, **kw)
        elif kind == "reduce":
            p = ff.make_plan(ff.FAMILY_REDUCE, bn2=128, raster=1, splits=(N1 + kw["bh"] - 1) // kw["bh"], **kw)
        else:
            p = ff.make_plan(ff.FAMILY_EXCHANGE, 256, 128 if gated else 256, bn2=256, raster=1, splits=1, **kw)
    eager = gu.run(w, dev, plan=p)                      # sizes the workspace, fills the plan table
    gu.check(eager, ref, "bf16", what="eager")
    Y = torch.zeros_like(eager)
    side = torch.cuda.Stream()
    ff.ffuse_force_plan(p)
    try:
        with torch.cuda.stream(side):
            ff.ffuse_ffn(dev["X"], dev["W1"], dev["W3"], dev["W2"], act, Y)      # warm-up on the capture stream
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                ff.ffuse_ffn(dev["X"], dev["W1"], dev["W3"], dev["W2"], act, Y)
        torch.cuda.synchronize()
        for rep in range(3):
            Y.fill_(float("nan"))
            scratch = torch.randn(1 << 20, device="cuda").sum()      # eager work between replays
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(Y, eager) or float((Y.float() - eager.float()).abs().max()) <= 2e-2 * float(eager.float().abs().max()), f"replay {rep}"
            gu.check(Y, ref, "bf16", what=f"replay {rep}")
            del scratch
        again = gu.run(w, dev, plan=p)                  # and the eager path still works afterwards
        gu.check(again, ref, "bf16", what="eager after replays")
    finally:
        ff.ffuse_force_plan(None)
