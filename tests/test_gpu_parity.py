"""Parity of the HIP path (through the C ABI) against the fp64 CPU oracle, on the same seeded
inputs.  Bar: max|Y - Y_ref| <= 2e-2 * max|Y_ref| for 16-bit operands, 1e-3 for fp32."""
import numpy as np
import pytest
import torch

from paper_2512_12949_amd import binding as ff
from paper_2512_12949_amd import inputs
from paper_2512_12949_amd.inputs import ACT_GELU_TANH, ACT_IDENTITY, ACT_RELU, ACT_SILU

import gpu_util as gu

pytestmark = pytest.mark.gpu

REDUCE_TILES = {False: [(256, 256), (128, 256), (128, 128), (128, 64)], True: [(256, 128), (128, 128), (128, 64)]}


def _case(name, M, K, N1, N2, dtype, act, gated, dist="normal", cfg_id=900):
    w = inputs.custom(name, M, K, N1, N2, dtype=dtype, act=act, gated=gated, dist=dist, cfg_id=cfg_id)
    host = inputs.make(w)
    dev = {k: gu.to_device(v, dtype) for k, v in host.items()}
    return w, host, dev


def test_tiny_fp32_config_fused_and_unfused():
    w = inputs.WORKLOADS["tiny"]
    host = inputs.make(w)
    dev = {k: gu.to_device(v, w.dtype) for k, v in host.items()}
    ref = gu.oracle_rows(w, host)
    print("tiny fused   rel err", gu.check(gu.run(w, dev), ref, "f32", what="tiny fused"), flush=True)
    print("tiny unfused rel err", gu.check(gu.run(w, dev, unfused=True), ref, "f32", what="tiny unfused"), flush=True)


@pytest.mark.parametrize("gated", [False, True])
@pytest.mark.parametrize("act", [ACT_RELU, ACT_GELU_TANH, ACT_SILU, ACT_IDENTITY])
def test_fp32_ragged(act, gated):
    w, host, dev = _case("f32r", 37, 72, 200, 40, "f32", act, gated)
    ref = gu.oracle_rows(w, host)
    gu.check(gu.run(w, dev), ref, "f32", what="f32 fused")
    gu.check(gu.run(w, dev, unfused=True), ref, "f32", what="f32 unfused")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("gated", [False, True])
def test_every_reduce_tile_on_a_ragged_shape(dtype, gated):
    """Several tiles in every dimension plus ragged tails in M, K, N1 and N2."""
    act = ACT_SILU if gated else ACT_GELU_TANH
    w, host, dev = _case("ragged", 300, 200, 328, 136, dtype, act, gated)
    ref = gu.oracle_rows(w, host)
    for bm, bh in REDUCE_TILES[gated]:
        for raster in (1, 2):
            plan = ff.make_plan(ff.FAMILY_REDUCE, bm, bh, raster=raster)
            print(f"ragged {dtype} gated={gated} tile {bm}x{bh} raster {raster}", flush=True)
            gu.check(gu.run(w, dev, plan=plan), ref, dtype, what=f"tile {bm}x{bh}")
    gu.check(gu.run(w, dev, unfused=True), ref, dtype, what="unfused")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("gated", [False, True])
def test_exchange_family_on_ragged_shapes(dtype, gated):
    """Producer/consumer ring kernel: ragged last panel, hidden tail, several panel groups,
    several producer counts and a ring small enough to wrap many times."""
    act = ACT_SILU if gated else ACT_GELU_TANH
    cases = [((600, 200, 840, 520), ((16, 32), (8, 20), (24, 8))),
             ((2300, 136, 392, 264), ((16, 32), (8, 28), (24, 12)))]
    for (M, K, N1, N2), settings in cases:
        w, host, dev = _case("exch", M, K, N1, N2, dtype, act, gated)
        ref = gu.oracle_rows(w, host)
        for producers, ring in settings:
            plan = ff.make_plan(ff.FAMILY_EXCHANGE, 256, 128 if gated else 256, bn2=256, producers=producers, ring=ring)
            print(f"exchange {dtype} gated={gated} shape {(M, K, N1, N2)} P={producers} R={ring}", flush=True)
            gu.check(gu.run(w, dev, plan=plan), ref, dtype, what=f"exchange P={producers} R={ring}")
        # the placement-independent protocol (agent-scope release/acquire)
        plan = ff.make_plan(ff.FAMILY_EXCHANGE, 256, 128 if gated else 256, bn2=256, producers=16, ring=32, coherent=1)
        gu.check(gu.run(w, dev, plan=plan), ref, dtype, what="exchange coherent")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("gated", [False, True])
def test_two_phase_small_m_family(dtype, gated):
    """Small-M kernel: every row padding (32 / 64 / 128), ragged K / N1 / N2, several splits,
    more hidden slices and output blocks than workgroups, and back-to-back launches that
    rely on the kernel leaving its barrier flags clean."""
    act = ACT_SILU if gated else ACT_GELU_TANH
    for (M, K, N1, N2) in [(1, 72, 136, 72), (16, 200, 840, 264), (50, 136, 392, 520), (128, 64, 33000, 136),
                           (7, 64, 256, 33000)]:
        w, host, dev = _case("small", M, K, N1, N2, dtype, act, gated)
        ref = gu.oracle_rows(w, host)
        for splits in (1, 3, 8):
            plan = ff.make_plan(ff.FAMILY_TWOPHASE, splits=splits)
            print(f"two-phase {dtype} gated={gated} shape {(M, K, N1, N2)} splits={splits}", flush=True)
            gu.check(gu.run(w, dev, plan=plan), ref, dtype, what=f"two-phase splits={splits}")
            gu.check(gu.run(w, dev, plan=plan), ref, dtype, what=f"two-phase splits={splits} again")
            deep = ff.make_plan(ff.FAMILY_TWOPHASE, bh=128, bk=32, splits=splits)   # LDS-direct loop, row block picked from M
            gu.check(gu.run(w, dev, plan=deep), ref, dtype, what=f"two-phase bk=32 splits={splits}")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("gated", [False, True])
def test_two_phase_family_with_row_blocks(dtype, gated):
    """Two-phase kernel beyond one row block: 128- and 256-row blocks, ragged last block,
    ragged K / N1 / N2, direct output (one range) and partial planes (several ranges), every
    raster, more work items than workgroups."""
    act = ACT_SILU if gated else ACT_GELU_TANH
    for (M, K, N1, N2) in [(300, 200, 840, 264), (1000, 136, 1304, 520), (2600, 72, 520, 776)]:
        w, host, dev = _case("blocks", M, K, N1, N2, dtype, act, gated)
        rows = inputs.sample_rows(M, 128, 24, seed=5)
        ref = gu.oracle_rows(w, host, rows)
        for bm, splits, raster in ((128, 1, 1), (128, 3, 2), (256, 1, 4), (256, 2, 8)):
            plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, splits=splits, raster=raster)
            print(f"two-phase {dtype} gated={gated} shape {(M, K, N1, N2)} bm={bm} splits={splits} raster={raster}", flush=True)
            gu.check(gu.run(w, dev, plan=plan), ref, dtype, rows=rows, what=f"two-phase bm={bm} splits={splits}")
            gu.check(gu.run(w, dev, plan=plan), ref, dtype, rows=rows, what=f"two-phase bm={bm} splits={splits} again")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("gated", [False, True])
def test_two_phase_narrow_hidden_slices(dtype, gated):
    """Phase-1 items of 64 and 32 hidden columns (2 x 2 waves, four waves along the rows):
    one row block and several, ragged everything."""
    act = ACT_SILU if gated else ACT_GELU_TANH
    for (M, K, N1, N2) in [(50, 136, 392, 520), (128, 200, 840, 264), (300, 72, 1304, 136)]:
        w, host, dev = _case("narrow", M, K, N1, N2, dtype, act, gated)
        ref = gu.oracle_rows(w, host)
        for bm, bh, splits in ((64, 64, 2), (128, 64, 1), (128, 64, 3), (128, 32, 1), (128, 32, 4)):
            if (bm < 128 and M > bm) or (bh == 32 and gated):
                continue
            plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=bh, splits=splits, raster=2)
            print(f"two-phase {dtype} gated={gated} shape {(M, K, N1, N2)} bm={bm} bh={bh} splits={splits}", flush=True)
            gu.check(gu.run(w, dev, plan=plan), ref, dtype, what=f"two-phase bm={bm} bh={bh} splits={splits}")
        for bm, bh, splits in ((64, 128, 2), (128, 128, 1), (128, 128, 3), (64, 64, 2), (128, 64, 1), (128, 64, 3)):
            if bm < 128 and M > bm:    # LDS-direct block GEMM on small row blocks (bk = 32), 128- and 64-column slices
                continue
            plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=bh, bk=32, splits=splits, raster=2)
            print(f"two-phase {dtype} gated={gated} shape {(M, K, N1, N2)} bm={bm} bh={bh} bk=32 splits={splits}", flush=True)
            gu.check(gu.run(w, dev, plan=plan), ref, dtype, what=f"two-phase bm={bm} bh={bh} bk=32 splits={splits}")
        for bm, bk in ((32, 64), (32, 32), (64, 64), (64, 32)):   # a few small row blocks instead of one large one
            if M > 4 * bm:
                continue
            plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=128, bk=bk, splits=2, raster=2)
            print(f"two-phase {dtype} gated={gated} shape {(M, K, N1, N2)} bm={bm} bk={bk} in {-(-M // bm)} row blocks", flush=True)
            gu.check(gu.run(w, dev, plan=plan), ref, dtype, what=f"two-phase bm={bm} bk={bk} row blocks")
    if gated:   # a 32-column slice cannot serve two weight matrices
        w, host, dev = _case("narrow", 128, 64, 256, 64, dtype, act, gated)
        with pytest.raises(ff.FfuseError):
            gu.run(w, dev, plan=ff.make_plan(ff.FAMILY_TWOPHASE, bm=128, bh=32, splits=1))


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("gated", [False, True])
def test_two_phase_non_temporal_weight_streaming(dtype, gated, monkeypatch):
    """The instantiations that stream the weights with the non-temporal hint (chosen by the
    library for weights far larger than the memory-side cache; forced here on small ragged
    shapes): every row block below 256 in both block GEMMs, and the same bits as without
    the hint."""
    act = ACT_SILU if gated else ACT_GELU_TANH
    for (M, K, N1, N2) in [(20, 136, 392, 520), (128, 200, 840, 264), (300, 72, 1304, 136)]:
        w, host, dev = _case("nt", M, K, N1, N2, dtype, act, gated)
        ref = gu.oracle_rows(w, host)
        for bm, bh, bk, splits in ((32, 128, 64, 2), (32, 128, 32, 2), (64, 128, 64, 1), (64, 64, 32, 3), (128, 128, 64, 1),
                                   (128, 128, 32, 2), (128, 64, 32, 3), (128, 64, 64, 1)):
            if M > 4 * bm and bm < 128:
                continue
            plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=bh, bk=bk, splits=splits, raster=2)
            print(f"non-temporal {dtype} gated={gated} shape {(M, K, N1, N2)} bm={bm} bh={bh} bk={bk} splits={splits}", flush=True)
            monkeypatch.setenv("FFUSE_NT", "0")
            plain = gu.run(w, dev, plan=plan)
            monkeypatch.setenv("FFUSE_NT", "1")
            hinted = gu.run(w, dev, plan=plan)
            gu.check(hinted, ref, dtype, what=f"non-temporal bm={bm} bh={bh} bk={bk}")
            assert torch.equal(plain, hinted)
    monkeypatch.delenv("FFUSE_NT")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("gated", [False, True])
def test_two_phase_256_row_tiles_with_several_items_per_workgroup(dtype, gated, monkeypatch):
    """256-row tiles where some workgroups own two first-phase items (286 items, ragged last row block and
    last hidden slice): the second item's ring fill is issued before the first item's epilogue and travels
    under it.  K shorter than the ring is deep, and longer; same bits with the fill behind the epilogue
    (FFUSE_EARLY_FILL=0)."""
    act = ACT_SILU if gated else ACT_GELU_TANH
    N1 = 3208 if gated else 6408
    for K in (8, 40, 72, 328):          # 1, 2 and 3 K steps (the ring is filled three steps deep), and 11
        w, host, dev = _case("fill", 2600, K, N1, 264, dtype, act, gated)
        rows = inputs.sample_rows(2600, 256, 6, seed=11)
        ref = gu.oracle_rows(w, host, rows)
        plans = [ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, splits=1, raster=4), ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, splits=2, raster=2)]
        for plan in plans:
            print(f"early fill {dtype} gated={gated} K={K} splits={plan.splits} raster={plan.raster}", flush=True)
            monkeypatch.setenv("FFUSE_EARLY_FILL", "1")
            early = gu.run(w, dev, plan=plan)
            gu.check(early, ref, dtype, rows=rows, what=f"early fill K={K} splits={plan.splits}")
            monkeypatch.setenv("FFUSE_EARLY_FILL", "0")
            late = gu.run(w, dev, plan=plan)
            assert torch.equal(early, late)
    monkeypatch.delenv("FFUSE_EARLY_FILL")


def test_two_launches_give_the_fused_calls_bits():
    """The unfused comparison path runs the fused kernel one phase per launch in the model's
    best two-phase plan: forced to that plan, the fused call must produce the same bits."""
    for (M, K, N1, N2, gated) in [(16, 520, 2056, 264, True), (128, 264, 4104, 520, False), (700, 136, 1304, 264, True)]:
        act = ACT_SILU if gated else ACT_GELU_TANH
        w, host, dev = _case("twolaunch", M, K, N1, N2, "bf16", act, gated)
        ref = gu.oracle_rows(w, host)
        two = gu.run(w, dev, unfused=True)
        gu.check(two, ref, "bf16", what="two launches")
        ranked = ff.ffuse_rank_plans(ff.DT_BF16, act, gated, M, K, N1, N2, 64)
        best = [p for p, _ in ranked if p.family == ff.FAMILY_TWOPHASE][0]
        print(f"two launches vs fused, shape {(M, K, N1, N2)} gated={gated}, plan {best.as_dict()}", flush=True)
        one = gu.run(w, dev, plan=best)
        assert torch.equal(one, two)


def test_group_local_barrier_gives_the_same_bits(monkeypatch):
    """Where every second-phase item of a workgroup group reads only what the group's own
    first-phase items wrote (ffuse_plan_group_local), the barrier between the phases waits for
    the group alone.  Same plan with the device-wide barrier: the same bits; both within
    tolerance of the oracle; repeated calls (the counters are left clean)."""
    cases = [(128, 520, 4096, 2048, False, ACT_GELU_TANH, 64, 128, 8, 2), (100, 264, 11008, 1032, True, ACT_SILU, 64, 128, 8, 2),
             (16, 1032, 7168, 520, True, ACT_SILU, 32, 128, 8, 1), (128, 136, 3072, 768, False, ACT_RELU, 64, 64, 16, 2),
             (2048, 264, 1024, 520, False, ACT_GELU_TANH, 256, 256, 1, 1), (1000, 136, 2048, 264, True, ACT_SILU, 128, 128, 1, 1),
             (700, 264, 4104, 520, False, ACT_GELU_TANH, 256, 256, 1, 4)]      # (the last one is not group-local)
    locals_seen = 0
    for n, (M, K, N1, N2, gated, act, bm, bh, splits, raster) in enumerate(cases):
        w, host, dev = _case("grp", M, K, N1, N2, "bf16", act, gated, cfg_id=720 + n)
        rows = None if M <= 256 else inputs.sample_rows(M, 256, 6, seed=n)
        ref = gu.oracle_rows(w, host, rows)
        plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=bh, bn2=256, bk=32, splits=splits, raster=raster)
        local = ff.ffuse_plan_group_local(plan, ff.DT_BF16, gated, M, K, N1, N2)
        locals_seen += int(local)
        print(f"group barrier: {(M, K, N1, N2)} gated={gated} plan {(bm, bh, splits, raster)} group-local={local}", flush=True)
        monkeypatch.setenv("FFUSE_GROUP_BARRIER", "1")
        outs = [gu.run(w, dev, plan=plan) for _ in range(3)]
        monkeypatch.setenv("FFUSE_GROUP_BARRIER", "0")
        wide = gu.run(w, dev, plan=plan)
        gu.check(outs[0], ref, "bf16", rows=rows, what="group-local barrier")
        gu.check(wide, ref, "bf16", rows=rows, what="device-wide barrier")
        for y in outs:
            assert torch.equal(y, wide)
    assert locals_seen >= 4
    monkeypatch.delenv("FFUSE_GROUP_BARRIER")


@pytest.mark.parametrize("act", [ACT_RELU, ACT_GELU_TANH, ACT_SILU, ACT_IDENTITY])
@pytest.mark.parametrize("gated", [False, True])
def test_activations_medium(act, gated):
    w, host, dev = _case("medium", 512, 512, 1024, 384, "bf16", act, gated)
    ref = gu.oracle_rows(w, host)
    print("medium fused  ", gu.check(gu.run(w, dev), ref, "bf16", what="fused"), flush=True)
    print("medium unfused", gu.check(gu.run(w, dev, unfused=True), ref, "bf16", what="unfused"), flush=True)


@pytest.mark.parametrize("shape", [(1, 8, 8, 8), (1, 64, 64, 64), (3, 16, 24, 8), (257, 264, 72, 520), (64, 8, 1032, 16)])
def test_degenerate_shapes(shape):
    M, K, N1, N2 = shape
    for gated in (False, True):
        w, host, dev = _case("edge", M, K, N1, N2, "bf16", ACT_SILU, gated)
        ref = gu.oracle_rows(w, host)
        gu.check(gu.run(w, dev), ref, "bf16", what=f"fused {shape}")
        gu.check(gu.run(w, dev, unfused=True), ref, "bf16", what=f"unfused {shape}")


def test_zero_weights_give_exact_zero():
    w, host, dev = _case("zero", 130, 64, 256, 128, "bf16", ACT_GELU_TANH, False)
    dev["W2"] = torch.zeros_like(dev["W2"])
    Y = gu.run(w, dev)
    assert torch.all(Y == 0)
    Y = gu.run(w, dev, unfused=True)
    assert torch.all(Y == 0)


def test_back_to_back_calls_share_one_workspace():
    """The fused call leaves its fp32 sums at zero; an unfused call in between dirties the
    workspace and the next fused call must still be right."""
    w, host, dev = _case("b2b", 200, 128, 512, 256, "bf16", ACT_RELU, False)
    ref = gu.oracle_rows(w, host)
    for i in range(3):
        gu.check(gu.run(w, dev), ref, "bf16", what=f"call {i}")
    gu.check(gu.run(w, dev, unfused=True), ref, "bf16", what="unfused between")
    gu.check(gu.run(w, dev), ref, "bf16", what="fused after unfused")


def test_workspace_errors_on_device():
    # a gated chain: every family that runs it needs a workspace (the rows family, which needs none, is not gated)
    w, host, dev = _case("ws", 64, 64, 64, 64, "bf16", ACT_SILU, True)
    Y = torch.empty((64, 64), dtype=torch.bfloat16, device="cuda")
    ff.ffuse_set_workspace(None)
    gu.Workspace.buf = None
    assert ff.ffuse_ffn(dev["X"], dev["W1"], dev["W3"], dev["W2"], ACT_SILU, Y, check=False) == -5
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    ff.ffuse_set_workspace(small)
    assert ff.ffuse_ffn(dev["X"], dev["W1"], dev["W3"], dev["W2"], ACT_SILU, Y, check=False) == -5
    ff.ffuse_set_workspace(None)


def test_tune_fills_the_plan_table_for_the_bin():
    """On-device tuning: the winner is one of the modelled candidates, later calls of the same M
    bin use it, other bins fall back to the model, and results stay within the parity bar."""
    ff.ffuse_plan_table_clear()
    w, host, dev = _case("tune", 200, 264, 1304, 520, "bf16", ACT_GELU_TANH, False)
    ref = gu.oracle_rows(w, host)
    gu.run(w, dev)                               # sizes and registers the workspace
    Y = torch.empty((200, 520), dtype=torch.bfloat16, device="cuda")
    plan, ms = ff.ffuse_tune(ff.DT_BF16, dev["X"], dev["W1"], None, dev["W2"], w.act, Y, top_k=5, reps=3)
    assert ms > 0 and plan.family in (ff.FAMILY_REDUCE, ff.FAMILY_EXCHANGE, ff.FAMILY_TWOPHASE, ff.FAMILY_ROWS)
    gu.check(Y, ref, "bf16", what="output left by tuning")
    looked, tuned_ms = ff.ffuse_plan_lookup(ff.DT_BF16, w.act, False, 200, 264, 1304, 520)
    assert looked.as_dict() == plan.as_dict() and tuned_ms == ms
    gu.check(gu.run(w, dev), ref, "bf16", what="fused call after tuning")
    assert ff.ffuse_last_plan().as_dict() == plan.as_dict()
    # same bin (129..256 rows), other M: the tuned plan when it is valid there
    looked2, _ = ff.ffuse_plan_lookup(ff.DT_BF16, w.act, False, 256, 264, 1304, 520)
    assert looked2.as_dict() == plan.as_dict()
    # another bin: the model's choice
    other, other_ms = ff.ffuse_plan_lookup(ff.DT_BF16, w.act, False, 64, 264, 1304, 520)
    assert other_ms == 0.0 and other.as_dict() == ff.ffuse_choose_plan(ff.DT_BF16, w.act, False, 64, 264, 1304, 520).as_dict()
    ff.ffuse_plan_table_clear()


def test_random_shapes_and_plans(monkeypatch):
    """Seeded random walk over valid shapes (ragged everything), operand types, activations and
    forced two-phase plans (row block, slice, block GEMM, hidden ranges, raster, weight-load
    hint), each against the oracle; the chooser's plan and the two-launch path ride along."""
    import random
    rng = random.Random(20251212)
    for n in range(40):
        M = rng.choice([1, 3, 16, 31, 33, 64, 65, 100, 128, 129, 200, 256, 300, 513, 700])
        K, N1, N2 = 8 * rng.randint(1, 80), 8 * rng.randint(1, 260), 8 * rng.randint(1, 90)
        gated, dtype, act = rng.random() < 0.5, rng.choice(["bf16", "f16"]), rng.choice([ACT_IDENTITY, ACT_RELU, ACT_GELU_TANH, ACT_SILU])
        w, host, dev = _case("random", M, K, N1, N2, dtype, act, gated, cfg_id=900 + n)
        ref = gu.oracle_rows(w, host)
        bm = rng.choice([32, 64, 128, 256])
        if bm < 128 and M > 4 * bm:
            bm = 128
        bh = (128 if gated else 256) if bm == 256 else (128 if bm < 64 else rng.choice([128, 64]))
        plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=bh, bk=rng.choice([32, 64]), splits=rng.choice([1, 2, 3, 5, 8]),
                            raster=rng.choice([1, 2, 4]))
        monkeypatch.setenv("FFUSE_NT", rng.choice(["0", "1"]))
        what = f"random {n}: {(M, K, N1, N2)} gated={gated} {dtype} act={act} plan={(plan.bm, plan.bh, plan.bk, plan.splits, plan.raster)}"
        print(what, flush=True)
        gu.check(gu.run(w, dev, plan=plan), ref, dtype, what=what)
        gu.check(gu.run(w, dev), ref, dtype, what=what + " (chooser)")
        gu.check(gu.run(w, dev, unfused=True), ref, dtype, what=what + " (two launches)")
    monkeypatch.delenv("FFUSE_NT")
