"""The entry point that allocates nothing (its workspace is device memory built into the library):
called through the C ABI twice in a row, the second time with a smaller input, and compared
with the ordinary entry point (caller-owned workspace) and with the oracle."""
import numpy as np
import pytest
import torch

from paper_2512_12949_amd import binding as ff
from paper_2512_12949_amd import inputs
from paper_2512_12949_amd.inputs import ACT_GELU_TANH, ACT_SILU

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _problem(name, M, K, N1, N2, gated, cfg_id):
    w = inputs.custom(name, M, K, N1, N2, dtype="bf16", act=ACT_SILU if gated else ACT_GELU_TANH, gated=gated, cfg_id=cfg_id)
    host = inputs.make(w)
    return w, host, {k: gu.to_device(v, "bf16") for k, v in host.items()}


def test_static_scratch_entry_point_two_calls_the_second_smaller():
    big = _problem("static-a", 128, 1032, 4104, 1032, True, 990)      # partial planes + intermediate + flags
    small = _problem("static-b", 50, 264, 840, 136, True, 991)        # smaller in every dimension: another layout in the same memory
    for w, host, dev in (big, small):
        print(f"static scratch: {(w.M, w.K, w.N1, w.N2)}", flush=True)
        Y = torch.full((w.M, w.N2), float("nan"), dtype=torch.bfloat16, device="cuda")
        ff.ffuse_ffn_static(ff.DT_BF16, dev["X"], dev["W1"], dev["W3"], dev["W2"], w.act, Y)
        assert ff.ffuse_sync_status(check=False) == 0
        torch.cuda.synchronize()
        want = gu.run(w, dev)                                           # the ordinary entry point, caller-owned workspace
        ref = gu.oracle_rows(w, host)
        gu.check(Y, ref, "bf16", what="static scratch vs oracle")
        gu.check(want, ref, "bf16", what="ordinary entry point vs oracle")
        scale = float(want.float().abs().max())
        assert float((Y.float() - want.float()).abs().max()) <= 2e-2 * scale
    # back to the larger problem: whatever the smaller one left in the memory is cleared by the call itself
    w, host, dev = big
    Y = torch.full((w.M, w.N2), float("nan"), dtype=torch.bfloat16, device="cuda")
    ff.ffuse_ffn_static(ff.DT_BF16, dev["X"], dev["W1"], dev["W3"], dev["W2"], w.act, Y)
    torch.cuda.synchronize()
    gu.check(Y, gu.oracle_rows(w, host), "bf16", what="static scratch, third call")


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    M, K, N1, N2 = 4096, 4096, 16384, 4096                              # needs 128 MiB for the intermediate
    X = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    W1 = torch.zeros((K, N1), dtype=torch.bfloat16, device="cuda")
    W2 = torch.zeros((N1, N2), dtype=torch.bfloat16, device="cuda")
    Y = torch.full((M, N2), 7.0, dtype=torch.bfloat16, device="cuda")
    assert ff.ffuse_ffn_static(ff.DT_BF16, X, W1, None, W2, 2, Y, check=False) == -5
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())                                       # nothing was written
    assert ff.ffuse_ffn_static(9, X, W1, None, W2, 2, Y, check=False) == -4
    # a shape the rows family runs needs no workspace at all: any size of it fits
    w, host, dev = _problem("static-rows", 20000, 520, 264, 520, False, 992)
    Yr = torch.full((w.M, w.N2), float("nan"), dtype=torch.bfloat16, device="cuda")
    ff.ffuse_ffn_static(ff.DT_BF16, dev["X"], dev["W1"], None, dev["W2"], w.act, Yr)
    torch.cuda.synchronize()
    rows = inputs.sample_rows(w.M, 256, 3, seed=3)
    gu.check(Yr, gu.oracle_rows(w, host, rows), "bf16", rows=rows, what="static scratch, large M")


def test_static_scratch_entry_point_recorded_into_a_graph():
    """What the entry point is for: after one eager call (which resolves the address of the built-in
    memory) a call is captured and replayed, with the input overwritten in place and with eager calls
    of other shapes using the same built-in memory between the replays."""
    w, host, dev = _problem("static-graph", 128, 520, 2056, 520, True, 993)
    hosts = [host] + [dict(host, X=inputs.make(inputs.custom("static-graph-x", w.M, w.K, w.N1, w.N2, dtype="bf16", act=w.act, gated=True,
                                                              cfg_id=994 + i))["X"]) for i in range(2)]
    refs = [gu.oracle_rows(w, h) for h in hosts]
    xs = [gu.to_device(h["X"], "bf16") for h in hosts]
    ow, ohost, odev = _problem("static-other", 77, 264, 840, 136, False, 997)
    oref = gu.oracle_rows(ow, ohost)
    X = xs[0].clone()
    Y = torch.zeros((w.M, w.N2), dtype=torch.bfloat16, device="cuda")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ff.ffuse_ffn_static(ff.DT_BF16, X, dev["W1"], dev["W3"], dev["W2"], w.act, Y)
        side.synchronize()
        gu.check(Y, refs[0], "bf16", what="eager")
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            ff.ffuse_ffn_static(ff.DT_BF16, X, dev["W1"], dev["W3"], dev["W2"], w.act, Y)
    torch.cuda.synchronize()
    for rep in range(5):
        i = (rep + 1) % 3
        X.copy_(xs[i])
        if rep % 2 == 1:
            Yo = torch.full((ow.M, ow.N2), float("nan"), dtype=torch.bfloat16, device="cuda")
            ff.ffuse_ffn_static(ff.DT_BF16, odev["X"], odev["W1"], None, odev["W2"], ow.act, Yo)
            torch.cuda.synchronize()
            gu.check(Yo, oref, "bf16", what="eager call of another shape between replays")
        Y.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        gu.check(Y, refs[i], "bf16", what=f"replay {rep} (input {i})")
