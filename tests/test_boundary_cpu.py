"""C-ABI boundary checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2512_12949_amd import binding as ff

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "ffuse.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ffuse_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 16
    L = ff.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(ff.EXPORTS) == names
    assert ff.ffuse_version() >= 1


def test_argument_validation_happens_before_any_device_work():
    L = ff.lib()
    a = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1008)
    call = L.ffuse_ffn
    assert call(None, a, None, a, 1, 8, 8, 8, 8, a, None) == -1
    assert call(a, a, None, a, 1, 8, 8, 8, 8, None, None) == -1
    assert call(a, a, None, a, 9, 8, 8, 8, 8, a, None) == -4
    assert call(a, a, None, a, 1, 0, 8, 8, 8, a, None) == -2
    assert call(a, a, None, a, 1, 8, 12, 8, 8, a, None) == -2
    assert call(a, a, None, a, 1, 8, 8, 4, 8, a, None) == -2
    assert call(a, a, None, a, 1, 1 << 20, 1 << 12, 8, 8, a, None) == -2   # X of 8 GiB
    assert call(odd, a, None, a, 1, 8, 8, 8, 8, a, None) == -3
    assert call(a, a, odd, a, 1, 8, 8, 8, 8, a, None) == -3
    for name in ("ffuse_ffn_f16", "ffuse_ffn_f32", "ffuse_ffn_unfused", "ffuse_ffn_unfused_f16", "ffuse_ffn_unfused_f32"):
        assert getattr(L, name)(None, a, None, a, 1, 8, 8, 8, 8, a, None) == -1
    assert ff.status_string(0) == "ok" and "NULL" in ff.status_string(-1)


def test_workspace_size_formula():
    # fused: the largest of the fp32 sums (reduce family), flags + 8 rings of 64 slots (exchange
    # family) and partial planes | H | flags (two-phase family; as many planes as fit in 64 MiB)
    def two_phase(M, N1, N2, planes):
        r = lambda v: (v + 255) // 256 * 256
        return (r(4 * M * N2 * planes) if planes > 1 else 0) + r(2 * M * N1) + 1024
    ring = 8192 + 8 * 64 * 256 * 256 * 2
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 4096, 4096, 16384, 4096, False) == max(4 * 4096 * 4096, ring, two_phase(4096, 16384, 4096, 1))
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 32768, 1024, 8192, 1024, False) == max(4 * 32768 * 1024, two_phase(32768, 8192, 1024, 1))
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 8192, 1024, 8192, 1024, False) == max(4 * 8192 * 1024, ring, two_phase(8192, 8192, 1024, 2))
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, True, 64, 64, 64, 64, False) == max(8192 + 8 * 64 * 256 * 128 * 2, two_phase(64, 64, 64, 32))
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 512, 4096, 16384, 4096, False) == max(ring, two_phase(512, 16384, 4096, 8))
    # unfused, 16-bit: the two-phase family's kernel, one phase per launch
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 4096, 4096, 16384, 4096, True) == two_phase(4096, 16384, 4096, 1)
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 512, 4096, 16384, 4096, True) == two_phase(512, 16384, 4096, 8)
    assert ff.ffuse_workspace_bytes(ff.DT_F32, False, 128, 256, 1024, 256, True) == 4 * 128 * 1024
    assert ff.ffuse_workspace_bytes(ff.DT_F32, False, 128, 256, 1024, 256, False) == 0


def test_plan_lookup_without_tuning_is_the_models_choice():
    ff.ffuse_plan_table_clear()
    for M in (1, 16, 17, 128, 300, 4096):
        want = ff.ffuse_choose_plan(ff.DT_BF16, 2, False, M, 4096, 16384, 4096).as_dict()
        got, tuned_ms = ff.ffuse_plan_lookup(ff.DT_BF16, 2, False, M, 4096, 16384, 4096)
        assert got.as_dict() == want and tuned_ms == 0.0
        again, _ = ff.ffuse_plan_lookup(ff.DT_BF16, 2, False, M, 4096, 16384, 4096)   # now from the table
        assert again.as_dict() == want
    ff.ffuse_plan_table_clear()


def test_tune_validates_before_touching_the_device():
    import ctypes
    L = ff.lib()
    p, ms = ff.Plan(), ctypes.c_double()
    rc = L.ffuse_tune(ff.DT_BF16, None, None, None, None, 2, 128, 64, 64, 64, None, 4, 3, None, ctypes.byref(p), ctypes.byref(ms))
    assert rc == -1
    rc = L.ffuse_tune(7, None, None, None, None, 2, 128, 64, 64, 64, None, 4, 3, None, ctypes.byref(p), ctypes.byref(ms))
    assert rc == -4


def test_plan_table_set_save_load_round_trip(tmp_path):
    ff.ffuse_plan_table_clear()
    plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=128, bh=64, bk=32, bn2=256, splits=4, h_level=2, raster=2)
    ff.ffuse_plan_table_set(ff.DT_BF16, False, 200, 4096, 16384, 4096, plan, ms=0.125)
    gated = ff.make_plan(ff.FAMILY_REDUCE, 128, 64, bn2=128, raster=1, splits=86)
    ff.ffuse_plan_table_set(ff.DT_F16, True, 16, 2048, 5632, 2048, gated, ms=0.05)
    got, ms = ff.ffuse_plan_lookup(ff.DT_BF16, 2, False, 256, 4096, 16384, 4096)      # same bin as M = 200
    assert got.as_dict() == plan.as_dict() and ms == 0.125
    other, ms0 = ff.ffuse_plan_lookup(ff.DT_BF16, 2, False, 64, 4096, 16384, 4096)    # another bin: the model
    assert ms0 == 0.0
    path = tmp_path / "plans.txt"
    assert ff.ffuse_plan_table_save(path) == 2                                         # modelled entries are not stored
    text = path.read_text().splitlines()
    assert len(text) == 2 and all(line.startswith("ffuse-plan 1 ") for line in text)
    ff.ffuse_plan_table_clear()
    assert ff.ffuse_plan_lookup(ff.DT_BF16, 2, False, 256, 4096, 16384, 4096)[1] == 0.0
    path.write_text(path.read_text() + "garbage line\nffuse-plan 9 0 0 1 1 1 1 1 1 1 1 1 1 1 1 1 1 1 1\n")
    assert ff.ffuse_plan_table_load(path) == 2                                         # bad lines are skipped
    got, ms = ff.ffuse_plan_lookup(ff.DT_BF16, 2, False, 130, 4096, 16384, 4096)
    assert got.as_dict() == plan.as_dict() and ms == 0.125
    got, ms = ff.ffuse_plan_lookup(ff.DT_F16, 3, True, 9, 2048, 5632, 2048)
    assert got.as_dict() == gated.as_dict() and ms == 0.05
    # an entry that is not valid for a concrete M of its bin is passed over at lookup time
    small = ff.make_plan(ff.FAMILY_TWOPHASE, bm=32, bh=128, bn2=256, splits=8, h_level=2, raster=1)
    ff.ffuse_plan_table_set(ff.DT_BF16, False, 20, 4096, 16384, 4096, small, ms=0.07)   # bin 17..32
    assert ff.ffuse_plan_lookup(ff.DT_BF16, 2, False, 32, 4096, 16384, 4096)[0].as_dict() == small.as_dict()
    bad = ff.Plan()
    assert ff.lib().ffuse_plan_table_set(ff.DT_BF16, 0, 100, 4096, 16384, 4096, __import__("ctypes").byref(bad), 1.0) == -8
    with pytest.raises(ff.FfuseError):
        ff.ffuse_plan_table_load(tmp_path / "missing.txt")
    ff.ffuse_plan_table_clear()


def test_ranked_plans_are_valid_sorted_and_fit_the_workspace_bound():
    """Host logic of the chooser (Sec. 4.3): everything it enumerates passes the model's own
    validity check, comes back sorted by predicted time, starts with what ffuse_choose_plan
    returns, and -- for the two-phase family, whose workspace depends on the plan -- fits what
    ffuse_workspace_bytes promises."""
    for (M, K, N1, N2, gated) in [(1, 4096, 16384, 4096, False), (16, 8192, 28672, 8192, True), (100, 4096, 11008, 4096, True),
                                  (128, 2048, 8192, 2048, False), (300, 1024, 4096, 1024, False), (2048, 4096, 11008, 4096, True),
                                  (4096, 4096, 16384, 4096, False)]:
        ranked = ff.ffuse_rank_plans(ff.DT_BF16, 2, gated, M, K, N1, N2, 1024)
        assert ranked, (M, K, N1, N2)
        times = [t for _, t in ranked]
        assert times == sorted(times)
        assert ranked[0][0].as_dict() == ff.ffuse_choose_plan(ff.DT_BF16, 2, gated, M, K, N1, N2).as_dict()
        bound = ff.ffuse_workspace_bytes(ff.DT_BF16, gated, M, K, N1, N2, False)
        for p, t in ranked:
            tr = ff.ffuse_traffic_model(p, ff.DT_BF16, gated, M, K, N1, N2).as_dict()   # raises on an invalid plan
            assert tr["feasible"] and t > 0
            if p.family == ff.FAMILY_TWOPHASE:
                r = lambda v: (v + 255) // 256 * 256
                need = (r(4 * M * N2 * p.splits) if p.splits > 1 else 0) + r(2 * M * N1) + 1024
                assert need <= bound, p.as_dict()


def test_streamed_weights_get_one_row_block():
    """Weights far larger than the memory-side cache are streamed with the non-temporal hint and
    are not kept for a second row block: below 256 rows per block the chooser must then cover
    all rows with one block (decode shapes), while cache-resident shapes may use two 64-row blocks."""
    for M in (16, 33, 64, 100, 128):
        p = ff.ffuse_choose_plan(ff.DT_BF16, 3, True, M, 8192, 28672, 8192)
        assert p.family == ff.FAMILY_TWOPHASE and (p.bm >= M or p.bm == 256), (M, p.as_dict())
    p = ff.ffuse_choose_plan(ff.DT_BF16, 2, False, 128, 2048, 8192, 2048)
    assert p.family == ff.FAMILY_TWOPHASE and p.bm in (64, 128)


def test_group_local_barrier_condition_matches_the_item_maps():
    """Host logic of the two-phase family's barrier scope: ffuse_plan_group_local must say 1
    exactly when every second-phase item of a workgroup group reads only tiles of the
    intermediate that first-phase items of the same group write.  Checked against an enumeration
    written here from the kernel's documented item map (items are dealt group by group, ceil(total/8)
    consecutive items each; within a group's range, patches of `raster` row blocks x all slices,
    row block fastest)."""
    import random

    def item(MB, S, raster, grp, idx):
        total = MB * S
        per = -(-total // 8)
        v = grp * per + idx
        if idx >= per or v >= total:
            return None
        panel, rem = divmod(v, raster * S)
        rows = min(raster, MB - panel * raster)
        return panel * raster + rem % rows, rem // rows

    def independent(M, N1, N2, bm, bh1, splits, raster):
        MB, NS1, NCB = -(-M // bm), -(-N1 // bh1), -(-N2 // 256)
        raster = min(raster, MB)
        ksplit = -(-(-(-N1 // splits)) // 64) * 64
        splits = -(-N1 // ksplit)
        owner = {}
        for g in range(8):
            idx = 0
            while (it := item(MB, NS1, raster, g, idx)) is not None:
                owner[it] = g
                idx += 1
        for g in range(8):
            idx = 0
            while (it := item(MB, NCB * splits, raster, g, idx)) is not None:
                rb, u = it
                sp = u // NCB
                k0, k1 = sp * ksplit, min(N1, (sp + 1) * ksplit)
                s = k0 // bh1
                while s * bh1 < k1:
                    if owner[(rb, s)] != g:
                        return False
                    s += 1
                idx += 1
        return True

    rng = random.Random(7)
    cases = [(4096, 4096, 16384, 4096, False, 256, 256, 1, 4), (4096, 4096, 16384, 4096, False, 256, 256, 1, 2),
             (2048, 4096, 11008, 4096, True, 256, 128, 2, 4), (2048, 4096, 11008, 4096, True, 256, 128, 2, 1),
             (32768, 1024, 8192, 1024, False, 256, 256, 1, 4), (16, 8192, 28672, 8192, True, 32, 128, 8, 1),
             (128, 4096, 16384, 4096, False, 64, 128, 8, 2), (128, 4096, 11008, 4096, True, 64, 128, 8, 2)]
    for _ in range(60):
        bm = rng.choice([32, 64, 128, 256])
        M = rng.randint(1, 4 * bm if bm < 128 else 2000)
        gated = rng.random() < 0.5
        bh1 = (128 if gated else 256) if bm == 256 else (128 if bm < 64 else rng.choice([128, 64]))
        cases.append((M, 8 * rng.randint(8, 64), 8 * rng.randint(1, 1500), 8 * rng.randint(1, 300), gated, bm, bh1,
                      rng.choice([1, 2, 3, 4, 8, 16]), rng.choice([1, 2, 4, 8])))
    seen = set()
    for (M, K, N1, N2, gated, bm, bh1, splits, raster) in cases:
        plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=bh1, bn2=256, bk=32, splits=splits, raster=raster)
        try:
            got = ff.ffuse_plan_group_local(plan, ff.DT_BF16, gated, M, K, N1, N2)
        except ff.FfuseError:
            continue        # not a plan the kernels implement for this shape
        want = independent(M, N1, N2, bm, bh1, splits, raster)
        assert got == want, (M, K, N1, N2, gated, bm, bh1, splits, raster, got, want)
        seen.add(got)
    assert seen == {True, False}
    # the benchmark configurations: gpt with four row blocks per patch is not, with two it is
    assert not ff.ffuse_plan_group_local(ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, bh=256, bn2=256, bk=32, splits=1, raster=4), ff.DT_BF16, False, 4096, 4096, 16384, 4096)
    assert ff.ffuse_plan_group_local(ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, bh=256, bn2=256, bk=32, splits=1, raster=2), ff.DT_BF16, False, 4096, 4096, 16384, 4096)

