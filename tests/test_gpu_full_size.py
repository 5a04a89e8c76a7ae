"""Parity at the benchmark configurations' full sizes, in the launch configurations the
benchmark times: the chooser's plan, and the plan the on-device tuning of the model's six
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
