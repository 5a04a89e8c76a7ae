"""The gated chain with its two branches on different workgroups (Sec. 4.1, gated FFN, the first
realisation: full-width single-branch tiles, joined by a Mul pass through the shared cache)
against the fp64 oracle and against the one-workgroup realisation, for every row-block size of
the two-phase family, ragged row counts, several hidden ranges, both operand types; inputs that
change call after call on one workspace (a stale line of either intermediate would show), and
the llama configuration at full size."""
import numpy as np
import pytest
import torch

from paper_2512_12949_amd import binding as ff
from paper_2512_12949_amd import inputs
from paper_2512_12949_amd.inputs import ACT_GELU_TANH, ACT_RELU, ACT_SILU

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _plan(bm, bh, split=1, **kw):
    return ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=bh, bn2=256, gate_split=split, **kw)


def _case(name, M, K, N1, N2, dtype, act=ACT_SILU, cfg_id=960):
    w = inputs.custom(name, M, K, N1, N2, dtype=dtype, act=act, gated=True, cfg_id=cfg_id)
    host = inputs.make(w)
    return w, host, {k: gu.to_device(v, dtype) for k, v in host.items()}


CASES = [  # (M, K, N1, N2), (bm, bh of the split plan, bh of its one-workgroup twin), splits, bk
    ((600, 264, 1344, 520), (256, 256, 128), 1, 32),
    ((777, 520, 1280, 264), (256, 256, 128), 2, 32),
    ((200, 264, 1344, 520), (128, 128, 128), 1, 64),
    ((130, 136, 832, 264), (128, 64, 64), 4, 64),
    ((100, 264, 640, 520), (64, 128, 128), 2, 64),
    ((100, 520, 704, 136), (64, 128, 128), 1, 32),
    ((17, 264, 1344, 264), (32, 128, 128), 8, 64),
    ((128, 512, 1024, 512), (128, 128, 128), 8, 32),
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_split_branches_match_the_oracle_and_the_one_workgroup_realisation(dtype):
    for n, (shape, (bm, bh, bh_twin), splits, bk) in enumerate(CASES):
        act = [ACT_SILU, ACT_GELU_TANH, ACT_RELU][n % 3]
        w, host, dev = _case("gate-split", *shape, dtype, act=act, cfg_id=960 + n)
        ref = gu.oracle_rows(w, host)
        print(f"gate split {dtype} {shape} bm {bm} bh {bh} splits {splits} bk {bk}", flush=True)
        Y = gu.run(w, dev, plan=_plan(bm, bh, 1, splits=splits, bk=bk, raster=2))
        last = ff.ffuse_last_plan()
        assert last.family == ff.FAMILY_TWOPHASE and last.gate_split == 1
        gu.check(Y, ref, dtype, what=f"split branches {shape}")
        twin = gu.run(w, dev, plan=_plan(bm, bh_twin, 0, splits=splits, bk=bk, raster=2))
        gu.check(twin, ref, dtype, what=f"one-workgroup twin {shape}")
        # the two realisations differ by the two extra roundings of the split one (each branch to the operand type)
        scale = float(twin.float().abs().max())
        assert float((Y.float() - twin.float()).abs().max()) <= 1.5e-2 * scale
        assert torch.equal(Y, gu.run(w, dev, plan=_plan(bm, bh, 1, splits=splits, bk=bk, raster=2))), "two runs, different bits"


def test_split_branches_with_inputs_that_change_every_call():
    """Same shape, plan and workspace, two different X in turn: a line of H or U left in a cache from the
    previous call (or from this call's first phase, on the XCD that did not rewrite it) would carry the
    other input's values."""
    shape = (700, 264, 1408, 520)
    wa, ha, da = _case("gs-a", *shape, "bf16", cfg_id=975)
    wb, hb, db = _case("gs-b", *shape, "bf16", cfg_id=976)
    db = dict(db, W1=da["W1"], W3=da["W3"], W2=da["W2"])
    hb = dict(hb, W1=ha["W1"], W3=ha["W3"], W2=ha["W2"])
    ra, rb = gu.oracle_rows(wa, ha), gu.oracle_rows(wb, hb)
    for plan in (_plan(256, 256, 1, bk=32, raster=2), _plan(128, 128, 1, splits=2, raster=1)):
        for i in range(6):
            w, dev, ref = (wa, da, ra) if i % 2 == 0 else (wb, db, rb)
            gu.check(gu.run(w, dev, plan=plan), ref, "bf16", what=f"call {i}")


def test_what_the_split_realisation_cannot_run_is_a_plan_error():
    w, host, dev = _case("gs-ragged", 128, 264, 520, 264, "bf16")          # N1 not a multiple of 64: tiles would share cache lines
    Y = torch.full((w.M, w.N2), 3.0, dtype=torch.bfloat16, device="cuda")
    gu.Workspace.ensure(1 << 24)
    try:
        ff.ffuse_force_plan(_plan(128, 128, 1))
        assert ff.ffuse_ffn(dev["X"], dev["W1"], dev["W3"], dev["W2"], w.act, Y, check=False) == -8
        assert ff.ffuse_ffn(dev["X"], dev["W1"], None, dev["W2"], w.act, Y, check=False) == -8      # not gated
        ff.ffuse_force_plan(ff.make_plan(ff.FAMILY_REDUCE, bm=128, bh=128, gate_split=1))
        assert ff.ffuse_ffn(dev["X"], dev["W1"], dev["W3"], dev["W2"], w.act, Y, check=False) == -8
        torch.cuda.synchronize()
        assert bool((Y == 3.0).all())
    finally:
        ff.ffuse_force_plan(None)


def test_split_branches_on_the_llama_configuration():
    w = inputs.WORKLOADS["llama"]
    host = inputs.make(w)
    dev = {k: gu.to_device(v, w.dtype) for k, v in host.items()}
    rows = inputs.sample_rows(w.M, 256, 3, seed=11)
    ref = gu.oracle_rows(w, host, rows)
    for plan in (_plan(256, 256, 1, bk=32, raster=4, splits=1), _plan(256, 256, 1, bk=32, raster=4, splits=2)):
        Y = gu.run(w, dev, plan=plan)
        gu.check(Y, ref, w.dtype, rows=rows, what="llama, split branches")


def test_an_expired_wait_at_either_rendezvous_of_the_split_realisation_leaves_cleanly():
    """The split realisation meets twice per launch.  With the host asking for an arrival that never
    comes, the first wait expires: the Mul pass and the second product are skipped, every workgroup
    leaves, the call reports the timeout and the next call is right."""
    w, host, dev = _case("gs-timeout", 300, 136, 832, 264, "bf16", cfg_id=980)
    ref = gu.oracle_rows(w, host)
    plan = _plan(128, 128, 1, splits=2, raster=2)
    gu.check(gu.run(w, dev, plan=plan), ref, "bf16", what="before")
    Y = torch.full((w.M, w.N2), float("nan"), dtype=torch.bfloat16, device="cuda")
    ff.ffuse_force_plan(plan)
    try:
        for rep in range(2):
            ff.ffuse_debug_barrier(1, 64)
            try:
                assert ff.ffuse_ffn(dev["X"], dev["W1"], dev["W3"], dev["W2"], w.act, Y, check=False) == 0
                assert ff.ffuse_sync_status(check=False) == -9
            finally:
                ff.ffuse_debug_barrier(0, 1 << 24)
            Y.fill_(float("nan"))
            assert ff.ffuse_ffn(dev["X"], dev["W1"], dev["W3"], dev["W2"], w.act, Y, check=False) == 0
            assert ff.ffuse_sync_status(check=False) == 0
            gu.check(Y, ref, "bf16", what=f"call after the expired wait ({rep})")
    finally:
        ff.ffuse_debug_barrier(0, 1 << 24)
        ff.ffuse_force_plan(None)


def test_split_realisation_in_a_replayed_graph_with_the_input_overwritten():
    shape = (600, 264, 1344, 520)
    ws_, hs = zip(*[(_case("gs-graph", *shape, "bf16", cfg_id=985 + i)[:2]) for i in range(3)])
    w = ws_[0]
    base = {k: gu.to_device(v, "bf16") for k, v in hs[0].items()}
    hosts = [dict(hs[0], X=h["X"]) for h in hs]
    refs = [gu.oracle_rows(w, h) for h in hosts]
    xs = [gu.to_device(h["X"], "bf16") for h in hosts]
    plan = _plan(256, 256, 1, bk=32, raster=2)
    gu.check(gu.run(w, base, plan=plan), refs[0], "bf16", what="eager")
    X = xs[0].clone()
    Y = torch.zeros((w.M, w.N2), dtype=torch.bfloat16, device="cuda")
    side = torch.cuda.Stream()
    ff.ffuse_force_plan(plan)
    try:
        with torch.cuda.stream(side):
            ff.ffuse_ffn(X, base["W1"], base["W3"], base["W2"], w.act, Y)
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                ff.ffuse_ffn(X, base["W1"], base["W3"], base["W2"], w.act, Y)
        torch.cuda.synchronize()
        for rep in range(5):
            i = (rep + 1) % 3
            X.copy_(xs[i])
            if rep % 2 == 1:       # the one-workgroup realisation runs eagerly in the same workspace between replays
                gu.check(gu.run(w, dict(base, X=xs[i]), plan=_plan(128, 128, 0, splits=2)), refs[i], "bf16", what="eager twin")
                ff.ffuse_force_plan(plan)
            Y.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            gu.check(Y, refs[i], "bf16", what=f"replay {rep} (input {i})")
    finally:
        ff.ffuse_force_plan(None)
