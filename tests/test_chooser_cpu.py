"""Host-side chooser and traffic model (no GPU): capacity constraints, bytes never below the
compulsory minimum, the paper's counting identities, plans that can actually run, and the
rules of the boundary that are decided before any device work."""
import ctypes
import itertools

import pytest

from paper_2512_12949_amd import binding as ff

SHAPES = [  # (M, K, N1, N2, dtype, gated)
    (128, 256, 1024, 256, ff.DT_BF16, False), (4096, 4096, 16384, 4096, ff.DT_BF16, False),
    (2048, 4096, 11008, 4096, ff.DT_BF16, True), (16, 8192, 28672, 8192, ff.DT_BF16, True),
    (64, 8192, 28672, 8192, ff.DT_BF16, True), (32768, 1024, 8192, 1024, ff.DT_F16, False),
    (128, 4096, 16384, 4096, ff.DT_BF16, False), (1, 64, 64, 64, ff.DT_BF16, False), (300, 200, 328, 136, ff.DT_F16, True),
    (8192, 512, 4096, 512, ff.DT_BF16, False), (20000, 1000, 520, 1016, ff.DT_F16, False), (50000, 264, 136, 136, ff.DT_BF16, False),
]


def test_every_ranked_plan_respects_the_capacities_and_the_compulsory_bytes():
    """Sec. 4.3, Eq. 3 (capacity of every level) for every plan the chooser ranks: LDS per workgroup
    within 160 KB, accumulators within 256 registers per lane; and no level's modelled volume
    below what the method itself must move (X, the weights and Y once)."""
    seen_families = set()
    for M, K, N1, N2, dt, gated in SHAPES:
        ranked = ff.ffuse_rank_plans(dt, 2, gated, M, K, N1, N2, 512)
        assert ranked, (M, K, N1, N2)
        times = [t for _, t in ranked]
        assert times == sorted(times)
        e, g = 2, (2 if gated else 1)
        q_min = e * (M * K + g * K * N1 + N1 * N2 + M * N2)
        for plan, t_pred in ranked:
            tr = ff.ffuse_traffic_model(plan, dt, gated, M, K, N1, N2)
            assert tr.feasible == 1
            assert tr.lds_used <= 160 * 1024, plan.as_dict()
            assert tr.acc_regs <= 256, plan.as_dict()
            assert tr.q_min == q_min and tr.q_unfused == q_min + 2 * e * M * N1
            assert tr.hbm_bytes >= q_min, plan.as_dict()
            assert tr.fabric_bytes >= 0.999 * q_min or plan.family == ff.FAMILY_REDUCE, plan.as_dict()
            assert tr.t_pred > 0 and abs(tr.t_pred - t_pred) < 1e-12
            seen_families.add(plan.family)
    assert {ff.FAMILY_REDUCE, ff.FAMILY_TWOPHASE, ff.FAMILY_EXCHANGE, ff.FAMILY_ROWS} <= seen_families


def test_the_intermediate_is_charged_to_hbm_when_it_cannot_stay_in_the_memory_side_cache():
    """The two-phase family writes the intermediate through and reads it back: 512 MiB of it cannot
    come back from a 256 MB cache (the unfused path is charged by the same rule); 128 MiB can."""
    large = ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, bh=256, bn2=256, bk=32, splits=1, raster=4)
    t = ff.ffuse_traffic_model(large, ff.DT_F16, False, 32768, 1024, 8192, 1024)
    assert t.hbm_bytes == t.q_unfused
    t = ff.ffuse_traffic_model(large, ff.DT_BF16, False, 4096, 4096, 16384, 4096)
    assert t.hbm_bytes == t.q_min
    rows = ff.make_plan(ff.FAMILY_ROWS, bm=64, bh=64)
    t = ff.ffuse_traffic_model(rows, ff.DT_F16, False, 32768, 1024, 8192, 1024)
    assert t.hbm_bytes == t.q_min and t.exchange_bytes == 0 and t.reduce_bytes == 0
    assert t.fabric_bytes < t.q_unfused                      # the family exists to move fewer bytes than the unfused path
    assert t.acc_regs == 256 and t.lds_used <= 160 * 1024


def test_model_is_monotone_in_the_rows():
    for fam_plan in (ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, bh=256, bn2=256, bk=32, splits=1, raster=4),
                     ff.make_plan(ff.FAMILY_ROWS, bm=64, bh=64)):
        last = 0.0
        for M in (4096, 8192, 16384, 32768, 65536):
            t = ff.ffuse_traffic_model(fam_plan, ff.DT_BF16, False, M, 1024, 8192, 1024)
            assert t.t_pred >= last and t.flops == 2 * M * 8192 * (1024 + 1024)
            last = t.t_pred


def test_counting_identities_of_the_search_space():
    """Table of spatial / temporal partitions (Sec. 4.3): C(4, s) (4 - s)! schedules with s spatial
    dimensions, 24 + 12 + 4 + 1 = 41 in all; checked against a brute-force enumeration."""
    dims = "mnkl"
    brute = {s: 0 for s in range(1, 5)}
    for s in range(1, 5):
        for spatial in itertools.combinations(dims, s):
            rest = [d for d in dims if d not in spatial]
            brute[s] += len(set(itertools.permutations(rest)))
    assert [brute[s] for s in range(1, 5)] == [24, 12, 4, 1]
    assert [ff.ffuse_loop_schedule_count(s) for s in range(1, 5)] == [24, 12, 4, 1]
    assert ff.ffuse_loop_schedule_count(0) == 41 == sum(brute.values())
    assert ff.ffuse_loop_schedule_count(5) == 0
    # the size of the unpruned space the paper quotes for M = 256, N = 16384, K = L = 4096
    space = 41 * 5 ** 4 * (256 // 16) * (16384 // 16) * (4096 // 16) * (4096 // 16)
    assert abs(space / 2.75e13 - 1) < 0.01


def test_shuffle_and_reduce_group_sizes():
    """Sec. 4.1, the two worked examples: cluster (2, 4, 2, 4) has shuffle groups of 2 blocks and 2
    groups to reduce; cluster (2, 4, 2, 8) has shuffle groups of 4 and nothing to reduce."""
    assert ff.ffuse_cluster_exchange(4, 2, 4) == (2, 2)
    assert ff.ffuse_cluster_exchange(4, 2, 8) == (4, 1)
    assert ff.ffuse_cluster_exchange(1, 1, 1) == (1, 1)
    with pytest.raises(ff.FfuseError):
        ff.ffuse_cluster_exchange(4, 2, 3)
    with pytest.raises(ff.FfuseError):
        ff.ffuse_cluster_exchange(3, 2, 4)


def test_rows_family_geometry():
    ok = ff.make_plan(ff.FAMILY_ROWS, bm=64, bh=64)
    L = ff.lib()
    t = ff.Traffic()
    call = lambda M, K, N1, N2, gated, plan=ok: L.ffuse_traffic_model(ctypes.byref(plan), ff.DT_BF16, int(gated), M, K, N1, N2, ctypes.byref(t))
    assert call(32768, 1024, 8192, 1024, False) == 0
    assert call(100, 8, 8, 8, False) == 0
    assert call(32768, 1032, 8192, 1024, False) == -8        # X no longer fits the registers
    assert call(32768, 1024, 8192, 1032, False) == -8        # the output block no longer fits the accumulators
    assert call(32768, 1024, 8192, 1024, True) == -8         # two accumulator sets of the first product do not fit
    assert call(32768, 1024, 8192, 1024, False, ff.make_plan(ff.FAMILY_ROWS, bm=128, bh=64)) == -8
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 32768, 1024, 8192, 1024, False) > 0   # (sized for every family)


def test_bytes_objective_prefers_the_rows_family_where_it_is_close_enough():
    ff.ffuse_plan_table_clear()
    try:
        shape = (32768, 1024, 8192, 1024)
        ff.ffuse_set_objective(ff.OBJECTIVE_BYTES)
        p, _ = ff.ffuse_plan_lookup(ff.DT_F16, 1, False, *shape)
        assert p.family == ff.FAMILY_ROWS
        tb = ff.ffuse_traffic_model(p, ff.DT_F16, False, *shape)
        ff.ffuse_set_objective(ff.OBJECTIVE_TIME)
        # the fastest plan by the model is a 256-row two-phase plan; the rows family is predicted within a few per
        # cent of it with less than half its fabric bytes, and such a near-tie goes to it under the time objective too
        fastest, t_fastest = ff.ffuse_rank_plans(ff.DT_F16, 1, False, *shape)[0]
        tq = ff.ffuse_traffic_model(fastest, ff.DT_F16, False, *shape)
        assert fastest.family == ff.FAMILY_TWOPHASE and fastest.bm == 256
        assert tq.t_pred <= tb.t_pred <= 1.06 * tq.t_pred and tb.fabric_bytes < 0.5 * tq.fabric_bytes
        q, _ = ff.ffuse_plan_lookup(ff.DT_F16, 1, False, *shape)
        assert q.family == ff.FAMILY_ROWS
        # where the family is clearly slower (short K and few output columns: smaller chunks, the same fixed part per
        # row block) the time objective keeps the fastest plan
        for other in ((32768, 512, 4096, 512), (65536, 256, 2048, 256), (128, 1024, 4096, 1024)):
            r, _ = ff.ffuse_plan_lookup(ff.DT_F16, 1, False, *other)
            assert r.family != ff.FAMILY_ROWS
        # a shape the family cannot run keeps the time plan under either objective
        ff.ffuse_set_objective(ff.OBJECTIVE_BYTES)
        g, _ = ff.ffuse_plan_lookup(ff.DT_BF16, 2, False, 4096, 4096, 16384, 4096)
        assert g.family == ff.FAMILY_TWOPHASE
        with pytest.raises(ff.FfuseError):
            ff.ffuse_set_objective(7)
    finally:
        ff.ffuse_set_objective(ff.OBJECTIVE_TIME)
        ff.ffuse_plan_table_clear()


HUGE = [(262144, 64, 8192, 64), (65536, 1024, 16384, 1024), (131072, 512, 16384, 512), (131072, 1024, 16384, 1024)]


def test_an_intermediate_of_2_gib_or_more_is_a_shape_error():
    """The kernels that keep the intermediate in the workspace address it with 32-bit offsets: a
    problem whose M x N1 intermediate reaches 2 GiB is refused by every entry point before any
    device work (dummy pointers are never dereferenced)."""
    L = ff.lib()
    a = ctypes.c_void_p(0x1000)
    for M, K, N1, N2 in HUGE:
        assert (M + 256) * N1 * 2 >= 1 << 31
        for name in ("ffuse_ffn", "ffuse_ffn_f16", "ffuse_ffn_unfused", "ffuse_ffn_unfused_f16"):
            assert getattr(L, name)(a, a, None, a, 1, M, K, N1, N2, a, None) == -2, (name, M, K, N1, N2)
        assert L.ffuse_ffn_ws(ff.DT_BF16, a, a, None, a, 1, M, K, N1, N2, a, a, 1 << 20, None) == -2
        assert L.ffuse_tune(ff.DT_BF16, a, a, None, a, 1, M, K, N1, N2, a, 4, 2, None, None, None) == -2
    # just below the limit the call gets past validation (and then fails for want of a device or a workspace)
    assert L.ffuse_ffn(a, a, None, a, 1, 32768, 1024, 8192, 1024, a, None) != -2


def test_the_chooser_never_returns_a_plan_that_cannot_run():
    """Whatever the shape -- including intermediates of 2 GiB and more, which the boundary refuses
    anyway -- the chosen plan is valid for the problem, and a two-phase plan is never chosen when its
    intermediate does not fit the 32-bit offsets of the kernel."""
    shapes = [(s[0], s[1], s[2], s[3]) for s in SHAPES] + HUGE + [(1 << 20, 8, 1024, 8), (500000, 64, 2048, 64)]
    for M, K, N1, N2 in shapes:
        for gated in (False, True):
            for objective in (ff.OBJECTIVE_TIME, ff.OBJECTIVE_BYTES):
                ff.ffuse_set_objective(objective)
                try:
                    p, _ = ff.ffuse_plan_lookup(ff.DT_BF16, 3, gated, M, K, N1, N2)
                finally:
                    ff.ffuse_set_objective(ff.OBJECTIVE_TIME)
                t = ff.Traffic()
                rc = ff.lib().ffuse_traffic_model(ctypes.byref(p), ff.DT_BF16, int(gated), M, K, N1, N2, ctypes.byref(t))
                assert rc == 0 and t.feasible == 1, (M, K, N1, N2, gated, p.as_dict())
                if p.family == ff.FAMILY_TWOPHASE:
                    assert (M + 256) * N1 * 2 < 1 << 31, (M, K, N1, N2, p.as_dict())
    ff.ffuse_plan_table_clear()
    # a forced two-phase plan for such a shape is not a valid plan
    big = ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, bh=256, bn2=256, bk=32, splits=1, raster=4)
    t = ff.Traffic()
    assert ff.lib().ffuse_traffic_model(ctypes.byref(big), ff.DT_BF16, 0, 131072, 1024, 16384, 1024, ctypes.byref(t)) == -8


def test_per_call_workspace_arguments_are_validated_first():
    L = ff.lib()
    a, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    for name in ("ffuse_ffn_ws", "ffuse_ffn_unfused_ws"):
        f = getattr(L, name)
        assert f(7, a, a, None, a, 1, 8, 8, 8, 8, a, a, 256, None) == -4          # unknown operand type
        assert f(ff.DT_BF16, None, a, None, a, 1, 8, 8, 8, 8, a, a, 256, None) == -1
        assert f(ff.DT_BF16, a, a, None, a, 1, 8, 12, 8, 8, a, a, 256, None) == -2
        assert f(ff.DT_BF16, a, a, None, a, 1, 8, 8, 8, 8, a, odd, 256, None) == -3   # workspace alignment
        assert f(ff.DT_BF16, a, a, None, a, 1, 8, 8, 8, 8, a, a, 250, None) == -2     # workspace size not a multiple of 16
        assert f(ff.DT_BF16, a, a, None, a, 1, 8, 8, 8, 8, a, None, 256, None) == -1  # a size without a buffer
    assert L.ffuse_debug_barrier(-1, 10) == -2 and L.ffuse_debug_barrier(0, 0) == -2
    assert L.ffuse_debug_barrier(0, 1 << 24) == 0


def test_split_gate_plans_are_valid_only_where_the_kernel_can_run_them():
    """Gated chain with its branches on different workgroups (Sec. 4.1): two-phase family only, gated only,
    hidden size a multiple of 64 (tiles of the two intermediates must not share cache lines); the
    workspace holds both intermediates; the model never prefers it to its one-workgroup twin."""
    import ctypes
    split = ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, bh=256, bn2=256, bk=32, gate_split=1)
    twin = ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, bh=128, bn2=256, bk=32)
    shape = (2048, 4096, 11008, 4096)
    t1 = ff.ffuse_traffic_model(split, ff.DT_BF16, True, *shape)
    t0 = ff.ffuse_traffic_model(twin, ff.DT_BF16, True, *shape)
    assert t1.feasible and t1.t_pred > t0.t_pred and t1.fabric_bytes == t0.fabric_bytes + 3 * 2 * 2048 * 11008
    t = ff.Traffic()
    L = ff.lib()
    assert L.ffuse_traffic_model(ctypes.byref(split), ff.DT_BF16, 0, *shape, ctypes.byref(t)) == -8          # not gated
    assert L.ffuse_traffic_model(ctypes.byref(split), ff.DT_BF16, 1, 2048, 4096, 11016, 4096, ctypes.byref(t)) == -8   # N1 % 64
    for fam in (ff.FAMILY_REDUCE, ff.FAMILY_EXCHANGE, ff.FAMILY_ROWS):
        other = ff.make_plan(fam, bm=128, bh=128, gate_split=1)
        assert L.ffuse_traffic_model(ctypes.byref(other), ff.DT_BF16, 1, *shape, ctypes.byref(t)) == -8
    bad = ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, bh=256, bn2=256, bk=32, gate_split=2)
    assert L.ffuse_traffic_model(ctypes.byref(bad), ff.DT_BF16, 1, *shape, ctypes.byref(t)) == -8
    # room for both intermediates
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, True, *shape) >= 2 * 2 * 2048 * 11008
    for shp in (shape, (128, 4096, 11008, 4096), (16, 8192, 28672, 8192)):
        ranked = ff.ffuse_rank_plans(ff.DT_BF16, 3, True, *shp)
        splits = [i for i, (p, _) in enumerate(ranked) if p.gate_split]
        assert len(splits) == 1 and splits[0] > 0 and ranked[0][0].gate_split == 0
        assert all(p.gate_split == 0 for p, _ in ff.ffuse_rank_plans(ff.DT_BF16, 2, False, *shp))


def test_the_shipped_plan_table_loads_and_every_entry_is_runnable():
    """The plan table measured offline on an MI355X (paper_2512_12949_amd/plans_mi355x.txt, written by
    paper_2512_12949_amd.tune_plans): it parses, it covers the benchmark configurations and the paper's
    m = 128 tables, every plan is valid for its shape, and a lookup returns it for any M of its bin."""
    from paper_2512_12949_amd import inputs
    ff.ffuse_plan_table_clear()
    try:
        n = ff.ffuse_load_shipped_plans()
        names = ["gpt", "llama", "large", "decode16", "decode64"] + [f"G{i}" for i in range(1, 11)] + [f"S{i}" for i in range(1, 9)]
        assert n == len(names)
        for name in names:
            w = inputs.WORKLOADS[name]
            dt = ff.DTYPE_CODE[w.dtype]
            plan, ms = ff.ffuse_plan_lookup(dt, w.act, w.gated, w.M, w.K, w.N1, w.N2)
            assert ms > 0.0, name                                    # a measured entry, not the model's choice
            t = ff.ffuse_traffic_model(plan, dt, w.gated, w.M, w.K, w.N1, w.N2)     # raises on a plan that is not valid here
            assert t.feasible and 0.3 * t.t_pred < ms * 1e-3 < 3.0 * t.t_pred, (name, ms, t.t_pred)
        # the bin of M, not the exact M: 100 rows share the 65..128 bin with the table's 128
        w = inputs.WORKLOADS["G8"]
        a, ms_a = ff.ffuse_plan_lookup(ff.DT_BF16, w.act, False, 100, w.K, w.N1, w.N2)
        b, ms_b = ff.ffuse_plan_lookup(ff.DT_BF16, w.act, False, 128, w.K, w.N1, w.N2)
        assert ms_a == ms_b > 0 and a.as_dict() == b.as_dict()
        _, ms_c = ff.ffuse_plan_lookup(ff.DT_BF16, w.act, False, 300, w.K, w.N1, w.N2)
        assert ms_c == 0.0
    finally:
        ff.ffuse_plan_table_clear()
