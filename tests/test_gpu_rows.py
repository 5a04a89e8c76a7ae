"""The rows family (row-stationary fused chain: X in registers, the output block in accumulators,
one activated chunk in LDS, no workspace) against the fp64 oracle: every kernel instantiation
(K <= 512 / 1024, N2 <= 512 / 1024, whole and ragged tiles), both operand types, every activation,
two row blocks per workgroup, run-to-run identical bits, and the `large` workload at full size."""
import numpy as np
import pytest
import torch

from paper_2512_12949_amd import binding as ff
from paper_2512_12949_amd import inputs
from paper_2512_12949_amd.inputs import ACT_GELU_TANH, ACT_IDENTITY, ACT_RELU, ACT_SILU

import gpu_util as gu

pytestmark = pytest.mark.gpu

ROWS = ff.make_plan(ff.FAMILY_ROWS, bm=64, bh=64)


def _case(name, M, K, N1, N2, dtype, act, cfg_id=930):
    w = inputs.custom(name, M, K, N1, N2, dtype=dtype, act=act, gated=False, cfg_id=cfg_id)
    host = inputs.make(w)
    dev = {k: gu.to_device(v, dtype) for k, v in host.items()}
    return w, host, dev


# whole tiles and ragged ones for each of the four instantiations (K <= 512 | 1024) x (N2 <= 512 | 1024)
SHAPES = [(64, 1024, 64, 1024), (200, 1024, 512, 1024), (333, 1000, 520, 1016), (130, 512, 200, 512), (700, 264, 136, 136),
          (1, 8, 8, 8), (65, 520, 72, 520), (300, 512, 1024, 1024), (129, 1024, 192, 512), (500, 776, 328, 264), (64, 16, 4104, 1024)]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_rows_family_on_whole_and_ragged_tiles(dtype):
    for n, (M, K, N1, N2) in enumerate(SHAPES):
        act = [ACT_RELU, ACT_GELU_TANH, ACT_SILU, ACT_IDENTITY][n % 4]
        w, host, dev = _case("rows", M, K, N1, N2, dtype, act, cfg_id=930 + n)
        ref = gu.oracle_rows(w, host)
        print(f"rows {dtype} shape {(M, K, N1, N2)} act {act}", flush=True)
        Y = gu.run(w, dev, plan=ROWS)
        assert ff.ffuse_last_plan().family == ff.FAMILY_ROWS
        gu.check(Y, ref, dtype, what=f"rows {(M, K, N1, N2)}")
        assert torch.equal(Y, gu.run(w, dev, plan=ROWS)), "two runs, different bits"


def test_rows_family_needs_no_workspace():
    w, host, dev = _case("rows-nows", 300, 512, 520, 264, "bf16", ACT_GELU_TANH)
    ref = gu.oracle_rows(w, host)
    Y = torch.full((w.M, w.N2), float("nan"), dtype=torch.bfloat16, device="cuda")
    ff.ffuse_force_plan(ROWS)
    try:
        ff.ffuse_ffn_ws(ff.DT_BF16, dev["X"], dev["W1"], None, dev["W2"], w.act, Y, None)
        ff.ffuse_sync_status()
        gu.check(Y, ref, "bf16", what="rows without a workspace")
        # what the family cannot run is a plan error, not a wrong answer
        g = inputs.custom("rows-g", 128, 256, 256, 256, dtype="bf16", act=ACT_SILU, gated=True)
        gdev = {k: gu.to_device(v, "bf16") for k, v in inputs.make(g).items()}
        Yg = torch.empty((128, 256), dtype=torch.bfloat16, device="cuda")
        assert ff.ffuse_ffn_ws(ff.DT_BF16, gdev["X"], gdev["W1"], gdev["W3"], gdev["W2"], g.act, Yg, None, check=False) == -8
    finally:
        ff.ffuse_force_plan(None)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_rows_family_two_row_blocks_per_workgroup_same_bits_every_run(dtype):
    """More row blocks than compute units (every workgroup walks the hidden dimension twice, the
    weight stream running on across the boundary) on a short hidden dimension, where the
    boundary comes round often.  The weight ring re-aims loads at a slot only once the wave's
    reads of it have delivered: any slip there shows as a block that differs between runs."""
    M = 64 * 2 * torch.cuda.get_device_properties(0).multi_processor_count
    w, host, dev = _case("rows-2rb", M, 1024, 256, 1024, dtype, ACT_IDENTITY)
    rows = inputs.sample_rows(M, 64, 2, seed=11)
    ref = gu.oracle_rows(w, host, rows)
    first = gu.run(w, dev, plan=ROWS)
    gu.check(first, ref, dtype, rows=rows, what="rows, two row blocks per workgroup")
    for rep in range(12):
        again = gu.run(w, dev, plan=ROWS)
        assert torch.equal(first, again), f"run {rep} differs in rows {((first != again).any(dim=1).nonzero().flatten() // 64).unique().tolist()[:8]} (blocks of 64)"


def test_rows_family_large_at_full_size():
    w = inputs.WORKLOADS["large"]
    print("[large] generating inputs", flush=True)
    host = inputs.make(w)
    dev = {k: gu.to_device(v, w.dtype) for k, v in host.items()}
    rows = inputs.sample_rows(w.M, 64, 1, seed=w.cfg_id)
    print(f"[large] oracle on {len(rows)} rows", flush=True)
    ref = gu.oracle_rows(w, host, rows)
    Y = gu.run(w, dev, plan=ROWS)
    rel = gu.check(Y, ref, w.dtype, rows=rows, what="large, rows family")
    assert bool(torch.isfinite(Y.float()).all())
    Y2 = gu.run(w, dev)                                        # the chooser's plan: the same answer to rounding
    scale = float(Y2.float().abs().max())
    diff = float((Y.float() - Y2.float()).abs().max())
    print(f"[large] rows family rel err {rel:.3e}; vs chooser's plan {diff / scale:.3e}", flush=True)
    assert diff <= 2 * gu.TOL[w.dtype] * scale
    # the bytes objective runs this family here
    ff.ffuse_plan_table_clear()
    ff.ffuse_set_objective(ff.OBJECTIVE_BYTES)
    try:
        Y3 = gu.run(w, dev)
        assert ff.ffuse_last_plan().family == ff.FAMILY_ROWS
        assert torch.equal(Y3, Y)
    finally:
        ff.ffuse_set_objective(ff.OBJECTIVE_TIME)
        ff.ffuse_plan_table_clear()
