"""The cross-workgroup protocols under conditions that parity on fixed inputs does not reach: inputs
that change from call to call on one workspace, graph replays whose inputs were overwritten in
place, a replay after another family has dirtied the workspace, a barrier whose bounded wait
is made to expire from the host, two streams with a workspace each, and a bounded litmus loop
over the two-phase barrier and the exchange ring."""
import numpy as np
import pytest
import torch

from paper_2512_12949_amd import binding as ff
from paper_2512_12949_amd import inputs
from paper_2512_12949_amd.inputs import ACT_GELU_TANH, ACT_RELU, ACT_SILU

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _plans(gated, N1):
    return {
        "two-phase direct": ff.make_plan(ff.FAMILY_TWOPHASE, bm=128, bh=128, bk=32, splits=1, raster=2),
        "two-phase planes": ff.make_plan(ff.FAMILY_TWOPHASE, bm=128, bh=64, bk=32, splits=4, raster=1),
        "two-phase 256": ff.make_plan(ff.FAMILY_TWOPHASE, bm=256, splits=2, raster=4),
        "reduce": ff.make_plan(ff.FAMILY_REDUCE, 128, 64, bn2=128, raster=1, splits=(N1 + 63) // 64),
        "exchange": ff.make_plan(ff.FAMILY_EXCHANGE, 256, 128 if gated else 256, bn2=256, raster=1, splits=1, producers=16, ring=32),
    }


def _variants(w, n):
    """n seeded versions of the same problem that differ in X only."""
    host = inputs.make(w)
    out = []
    for i in range(n):
        wi = inputs.custom(w.name, w.M, w.K, w.N1, w.N2, dtype=w.dtype, act=w.act, gated=w.gated, cfg_id=w.cfg_id + 50 * (i + 1))
        hi = dict(host)
        hi["X"] = inputs.make(wi)["X"]
        out.append(hi)
    return out


@pytest.mark.parametrize("gated", [False, True])
def test_inputs_that_change_from_call_to_call(gated):
    """The two-phase barrier takes no cache invalidate; the intermediate of the previous call lies in
    the same workspace lines.  Alternating inputs call after call, every output must be the
    output of ITS input."""
    act = ACT_SILU if gated else ACT_GELU_TANH
    w = inputs.custom("alt", 700, 264, 1304, 520, dtype="bf16", act=act, gated=gated, cfg_id=940)
    hosts = _variants(w, 3)
    refs = [gu.oracle_rows(w, h) for h in hosts]
    devs = [{k: gu.to_device(v, "bf16") for k, v in h.items()} for h in hosts]
    for name, plan in _plans(gated, w.N1).items():
        print(f"alternating inputs, {name}, gated={gated}", flush=True)
        for rep in range(9):
            i = (rep * 2 + rep // 3) % 3
            Y = gu.run(w, devs[i], plan=plan)
            gu.check(Y, refs[i], "bf16", what=f"{name} call {rep} (input {i})")


@pytest.mark.parametrize("kind", ["two-phase direct", "two-phase planes", "two-phase 256", "reduce", "exchange", "rows"])
def test_graph_replays_with_inputs_overwritten_in_place(kind):
    """A captured call is replayed after its input buffer was overwritten in place and after an eager
    call of ANOTHER family has used (and dirtied) the same workspace: every replay must give the
    output of the input it found."""
    gated = False
    w = inputs.custom("gr", 600, 264, 1304, 520, dtype="bf16", act=ACT_GELU_TANH, gated=gated, cfg_id=950)
    hosts = _variants(w, 3)
    refs = [gu.oracle_rows(w, h) for h in hosts]
    devs = [{k: gu.to_device(v, "bf16") for k, v in h.items()} for h in hosts]
    plans = _plans(gated, w.N1)
    plans["rows"] = ff.make_plan(ff.FAMILY_ROWS, bm=64, bh=64)
    plan = plans[kind]
    other = plans["reduce" if kind != "reduce" else "two-phase planes"]
    gu.check(gu.run(w, devs[0], plan=plan), refs[0], "bf16", what="eager")       # sizes the workspace
    X = devs[0]["X"].clone()
    Y = torch.zeros((w.M, w.N2), dtype=torch.bfloat16, device="cuda")
    side = torch.cuda.Stream()
    ff.ffuse_force_plan(plan)
    try:
        with torch.cuda.stream(side):
            ff.ffuse_ffn(X, devs[0]["W1"], None, devs[0]["W2"], w.act, Y)          # warm-up on the capture stream
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                ff.ffuse_ffn(X, devs[0]["W1"], None, devs[0]["W2"], w.act, Y)
        torch.cuda.synchronize()
        for rep in range(6):
            i = (rep + 1) % 3
            X.copy_(devs[i]["X"])
            if rep % 2 == 1:                      # another family runs in the same workspace between replays
                gu.check(gu.run(w, devs[i], plan=other), refs[i], "bf16", what="eager call of the other family")
                ff.ffuse_force_plan(plan)
            Y.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            gu.check(Y, refs[i], "bf16", what=f"{kind} replay {rep} (input {i})")
    finally:
        ff.ffuse_force_plan(None)


def test_a_barrier_wait_that_expires_is_reported_and_does_not_poison_the_next_call():
    """The host asks the barrier to wait for one arrival more than there are workgroups and to give
    up after a few polls: every workgroup's bounded wait expires, every workgroup leaves normally,
    the call reports FFUSE_ERR_TIMEOUT -- and the very next call, with the hook off, is right."""
    w = inputs.custom("timeout", 300, 136, 840, 264, dtype="bf16", act=ACT_GELU_TANH, gated=False, cfg_id=960)
    host = inputs.make(w)
    dev = {k: gu.to_device(v, "bf16") for k, v in host.items()}
    ref = gu.oracle_rows(w, host)
    plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=128, splits=2, raster=2)
    gu.check(gu.run(w, dev, plan=plan), ref, "bf16", what="before")
    Y = torch.full((w.M, w.N2), float("nan"), dtype=torch.bfloat16, device="cuda")
    ff.ffuse_force_plan(plan)
    try:
        for rep in range(2):
            ff.ffuse_debug_barrier(1, 64)
            try:
                assert ff.ffuse_ffn(dev["X"], dev["W1"], None, dev["W2"], w.act, Y, check=False) == 0
                assert ff.ffuse_sync_status(check=False) == -9
            finally:
                ff.ffuse_debug_barrier(0, 1 << 24)
            Y.fill_(float("nan"))
            assert ff.ffuse_ffn(dev["X"], dev["W1"], None, dev["W2"], w.act, Y, check=False) == 0
            assert ff.ffuse_sync_status(check=False) == 0
            gu.check(Y, ref, "bf16", what=f"call after the expired wait ({rep})")
    finally:
        ff.ffuse_debug_barrier(0, 1 << 24)
        ff.ffuse_force_plan(None)
    gu.check(gu.run(w, dev, plan=plan), ref, "bf16", what="after")


def test_two_streams_with_a_workspace_each():
    """Calls that overlap in time on two streams, each with its own workspace passed per call."""
    ws_, hs, ds, refs, Ys, bufs = [], [], [], [], [], []
    for i, (M, K, N1, N2, gated) in enumerate([(700, 264, 2056, 520, False), (600, 136, 1304, 264, True)]):
        w = inputs.custom(f"s{i}", M, K, N1, N2, dtype="bf16", act=ACT_SILU if gated else ACT_RELU, gated=gated, cfg_id=970 + i)
        h = inputs.make(w)
        ws_.append(w); hs.append(h); ds.append({k: gu.to_device(v, "bf16") for k, v in h.items()})
        refs.append(gu.oracle_rows(w, h))
        Ys.append(torch.full((M, N2), float("nan"), dtype=torch.bfloat16, device="cuda"))
        need = ff.ffuse_workspace_bytes(ff.DT_BF16, gated, M, K, N1, N2, False)
        bufs.append(torch.empty(need, dtype=torch.uint8, device="cuda").fill_(0xA5))     # dirty on purpose
    ff.ffuse_set_workspace(None)
    gu.Workspace.buf = None
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(6):
        for i in (0, 1):
            with torch.cuda.stream(streams[i]):
                ff.ffuse_ffn_ws(ff.DT_BF16, ds[i]["X"], ds[i]["W1"], ds[i]["W3"], ds[i]["W2"], ws_[i].act, Ys[i], bufs[i],
                                stream=streams[i].cuda_stream)
        if rep % 2:
            for s in streams:
                s.synchronize()
            for i in (0, 1):
                gu.check(Ys[i], refs[i], "bf16", what=f"stream {i} round {rep}")
                Ys[i].fill_(float("nan"))
    torch.cuda.synchronize()
    # the two-launch path with a per-call workspace as well
    ff.ffuse_ffn_unfused_ws(ff.DT_BF16, ds[0]["X"], ds[0]["W1"], None, ds[0]["W2"], ws_[0].act, Ys[0], bufs[0])
    torch.cuda.synchronize()
    gu.check(Ys[0], refs[0], "bf16", what="two launches, per-call workspace")
    # a workspace that is too small is an error, not a fault
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    ff.ffuse_force_plan(ff.make_plan(ff.FAMILY_TWOPHASE, bm=128, splits=1, raster=1))
    try:
        assert ff.ffuse_ffn_ws(ff.DT_BF16, ds[0]["X"], ds[0]["W1"], None, ds[0]["W2"], ws_[0].act, Ys[0], small, check=False) == -5
    finally:
        ff.ffuse_force_plan(None)


@pytest.mark.parametrize("kind", ["two-phase planes", "two-phase 256", "exchange"])
def test_litmus_loop_over_the_flag_protocols(kind):
    """300 calls in a row on one workspace, the input changing every call, compared bit for bit with
    the output the same plan gave for that input in a first, oracle-checked round; stops at the
    first mismatch.  (The barrier counters, the ring's ready / done flags and the slots of the ring
    are reused by every call.)"""
    w = inputs.custom("litmus", 520, 136, 1304, 264, dtype="bf16", act=ACT_GELU_TANH, gated=False, cfg_id=980)
    hosts = _variants(w, 4)
    devs = [{k: gu.to_device(v, "bf16") for k, v in h.items()} for h in hosts]
    plan = _plans(False, w.N1)[kind]
    want = []
    for h, d in zip(hosts, devs):
        Y = gu.run(w, d, plan=plan)
        gu.check(Y, gu.oracle_rows(w, h), "bf16", what=f"{kind} reference round")
        want.append(Y.clone())
    Y = torch.empty_like(want[0])
    ff.ffuse_force_plan(plan)
    try:
        rng = np.random.default_rng(7)
        order = rng.integers(0, 4, size=300)
        for n, i in enumerate(order):
            ff.ffuse_ffn(devs[i]["X"], devs[i]["W1"], None, devs[i]["W2"], w.act, Y)
            if n % 25 == 24 or n == len(order) - 1:
                assert ff.ffuse_sync_status(check=False) == 0, f"{kind}: status after call {n}"
                assert torch.equal(Y, want[i]), f"{kind}: call {n} (input {i}) differs from the reference round"
    finally:
        ff.ffuse_force_plan(None)


def test_seeded_walk_over_every_family():
    """Bounded seeded walk over shapes, operand types, activations and plans of EVERY family (reduce,
    exchange, two-phase in both gated realisations, rows) against the oracle, all on one workspace."""
    import random
    rng = random.Random(20260101)
    for n in range(44):
        fam = rng.choice(["reduce", "exchange", "two", "rows"]) if n < 36 else "split"
        gated = (rng.random() < 0.5 and fam != "rows") or fam == "split"
        dtype, act = rng.choice(["bf16", "f16"]), rng.choice([0, 1, 2, 3])
        M = rng.choice([1, 33, 64, 130, 257, 520, 900])
        K, N1, N2 = 8 * rng.randint(1, 64), 8 * rng.randint(1, 200), 8 * rng.randint(1, 80)
        if fam == "split":       # the gated chain with its branches on different workgroups: hidden size in whole cache lines
            N1 = 64 * rng.randint(1, 25)
            bm = rng.choice([128, 256]) if M > 64 else rng.choice([32, 64, 128])
            if bm == 32 and M > 128:
                bm = 128
            plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=256 if bm == 256 else 128, bn2=256, bk=rng.choice([32, 64]),
                                splits=rng.choice([1, 2, 3]), raster=rng.choice([1, 2]), gate_split=1)
            fam = "two-split"
        if fam == "two-split":
            pass
        elif fam == "reduce":
            bm, bh = rng.choice([(256, 128), (128, 128), (128, 64)] if gated else [(256, 256), (128, 256), (128, 128), (128, 64)])
            plan = ff.make_plan(ff.FAMILY_REDUCE, bm, bh, bn2=128, raster=rng.choice([1, 2]), splits=(N1 + bh - 1) // bh)
        elif fam == "exchange":
            M = max(M, 257)
            producers = rng.choice([8, 16, 24])
            panels = (32 - producers) // -(-N2 // 256)                  # panels in flight per XCD group
            plan = ff.make_plan(ff.FAMILY_EXCHANGE, 256, 128 if gated else 256, bn2=256, raster=1, splits=1,
                                producers=producers, ring=max(rng.choice([12, 32, 64]), 2 * panels + 2))
        elif fam == "two":
            bm = rng.choice([128, 256])
            plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=(128 if gated else 256) if bm == 256 else rng.choice([128, 64]),
                                bk=rng.choice([32, 64]), splits=rng.choice([1, 2, 5]), raster=rng.choice([1, 2, 4]))
        else:
            plan = ff.make_plan(ff.FAMILY_ROWS, bm=64, bh=64)
        w = inputs.custom("walk", M, K, N1, N2, dtype=dtype, act=act, gated=gated, cfg_id=1000 + n)
        host = inputs.make(w)
        dev = {k: gu.to_device(v, dtype) for k, v in host.items()}
        what = f"walk {n}: {fam} {(M, K, N1, N2)} gated={gated} {dtype} act={act}"
        print(what, flush=True)
        gu.check(gu.run(w, dev, plan=plan), gu.oracle_rows(w, host), dtype, what=what)
