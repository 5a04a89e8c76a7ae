"""Parity at the benchmark configurations' full sizes (and at the paper's own m = 128 shape
tables), in the launch configurations the benchmark times: the chooser's plan, and the plan the on-device tuning of the model's six
best candidates settles on (what bench.py runs by default).  The oracle computes a stratified row sample (first,
last and seeded interior rows of every 256-row block; every output column), and the whole
output is checked for finiteness and against the unfused path."""
import numpy as np
import pytest
import torch

from paper_2512_12949_amd import binding as ff
from paper_2512_12949_amd import inputs

import gpu_util as gu

pytestmark = pytest.mark.gpu

PER_BLOCK = {"gpt": 4, "llama": 4, "decode16": 16, "decode64": 64, "large": 3}


@pytest.mark.parametrize("name", ["gpt", "llama", "decode16", "decode64", "large"])
def test_full_size(name):
    w = inputs.WORKLOADS[name]
    print(f"[{name}] generating inputs", flush=True)
    host = inputs.make(w)
    dev = {k: gu.to_device(v, w.dtype) for k, v in host.items()}
    rows = inputs.sample_rows(w.M, 256, PER_BLOCK[name], seed=w.cfg_id)
    print(f"[{name}] oracle on {len(rows)} rows", flush=True)
    ref = gu.oracle_rows(w, host, rows)
    print(f"[{name}] fused", flush=True)
    Y = gu.run(w, dev)
    plan = ff.ffuse_last_plan().as_dict()
    rel = gu.check(Y, ref, w.dtype, rows=rows, what=f"{name} fused")
    print(f"[{name}] fused plan {plan} rel err {rel:.3e}", flush=True)
    assert bool(torch.isfinite(Y.float()).all())
    print(f"[{name}] tuning the top 6 plans", flush=True)
    ff.ffuse_plan_table_clear()
    Yt = torch.full_like(Y, float("nan"))
    tuned, ms = ff.ffuse_tune(ff.DTYPE_CODE[w.dtype], dev["X"], dev["W1"], dev["W3"], dev["W2"], w.act, Yt, top_k=6, reps=3)
    Yt.fill_(float("nan"))
    ff.FUSED[w.dtype](dev["X"], dev["W1"], dev["W3"], dev["W2"], w.act, Yt)
    ff.ffuse_sync_status()
    assert ff.ffuse_last_plan().as_dict() == tuned.as_dict()
    relt = gu.check(Yt, ref, w.dtype, rows=rows, what=f"{name} tuned")
    print(f"[{name}] tuned plan {tuned.as_dict()} ({ms * 1e3:.1f} us) rel err {relt:.3e}", flush=True)
    assert bool(torch.isfinite(Yt.float()).all())
    ff.ffuse_plan_table_clear()
    print(f"[{name}] unfused", flush=True)
    Yu = gu.run(w, dev, unfused=True)
    relu = gu.check(Yu, ref, w.dtype, rows=rows, what=f"{name} unfused")
    scale = float(Yu.float().abs().max())
    diff = float((Y.float() - Yu.float()).abs().max())
    print(f"[{name}] unfused rel err {relu:.3e}; fused vs unfused {diff / scale:.3e}", flush=True)
    assert diff <= 2 * gu.TOL[w.dtype] * scale


TABLE_NAMES = [f"G{i}" for i in range(1, 11)] + [f"S{i}" for i in range(1, 9)]


@pytest.mark.parametrize("name", TABLE_NAMES)
def test_paper_shape_tables(name):
    """The paper's own shapes (Evaluation, tables of GEMM-chain and gated-FFN configurations, all
    at m = 128) at full size, in the chooser's plan and in the two-launch comparison path; the
    oracle computes a stratified row sample (every 32-row block's first and last row plus seeded
    interior rows, every output column).  A second call with fewer rows (M = 100: the same bin
    of the plan table, 65..128) is checked as well."""
    w = inputs.WORKLOADS[name]
    host = inputs.make(w)
    dev = {k: gu.to_device(v, w.dtype) for k, v in host.items()}
    rows = inputs.sample_rows(w.M, 32, 4, seed=w.cfg_id)
    ref = gu.oracle_rows(w, host, rows)
    Y = gu.run(w, dev)
    plan = ff.ffuse_last_plan().as_dict()
    rel = gu.check(Y, ref, w.dtype, rows=rows, what=f"{name} fused")
    assert bool(torch.isfinite(Y.float()).all())
    Yu = gu.run(w, dev, unfused=True)
    relu = gu.check(Yu, ref, w.dtype, rows=rows, what=f"{name} two launches")
    print(f"[{name}] {(w.M, w.K, w.N1, w.N2)} plan {plan} rel err {rel:.3e} (two launches {relu:.3e})", flush=True)
    # fewer rows, same bin: rows are independent, so the first 100 rows of Y are the answer
    dev100 = dict(dev)
    dev100["X"] = dev["X"][:100].contiguous()
    Y100 = gu.run(w, dev100)
    keep = rows[rows < 100]
    gu.check(Y100, ref[: len(keep)], w.dtype, rows=keep, what=f"{name} fused, 100 rows")


def test_shipped_plan_table_plans_run_and_match():
    """With the shipped plan table loaded, a call on a listed shape runs the table's plan (no tuning launches), and
    that plan's output meets the parity bar on the oracle's row sample -- the paper's m = 128 tables and the
    decode configurations (the three large configurations' tuned plans are covered by test_full_size)."""
    ff.ffuse_plan_table_clear()
    try:
        assert ff.ffuse_load_shipped_plans() >= 23
        for name in ["decode16", "decode64"] + TABLE_NAMES:
            w = inputs.WORKLOADS[name]
            host = inputs.make(w)
            dev = {k: gu.to_device(v, w.dtype) for k, v in host.items()}
            rows = inputs.sample_rows(w.M, 32, 2, seed=w.cfg_id)
            ref = gu.oracle_rows(w, host, rows)
            want, ms = ff.ffuse_plan_lookup(ff.DTYPE_CODE[w.dtype], w.act, w.gated, w.M, w.K, w.N1, w.N2)
            assert ms > 0.0, name
            Y = gu.run(w, dev)
            assert ff.ffuse_last_plan().as_dict() == want.as_dict(), name
            rel = gu.check(Y, ref, w.dtype, rows=rows, what=f"{name} shipped plan")
            assert bool(torch.isfinite(Y.float()).all())
            print(f"[{name}] shipped plan {want.as_dict()} ({ms * 1e3:.1f} us when tuned) rel err {rel:.3e}", flush=True)
    finally:
        ff.ffuse_plan_table_clear()
