"""Parity of the convolution-chain entry points (through the C ABI) against the fp64 CPU
oracle on the same seeded inputs: the paper's C1-C8 shapes in full, and small ragged cases
(batch > 1, image sides that are no multiple of anything, channel tails, single pixels)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_12949_amd import binding as ff
from paper_2512_12949_amd import inputs
from paper_2512_12949_amd.inputs import ACT_GELU_TANH, ACT_RELU, ACT_SILU

import gpu_util as gu

pytestmark = pytest.mark.gpu


def run_conv(w, host, plan=None):
    dt = ff.DTYPE_CODE[w.dtype]
    M, K, N1, N2 = w.gemm_shape()
    need = ff.ffuse_workspace_bytes(dt, False, M, K, N1, N2, False)
    if plan is not None:
        need = max(need, 4 * M * N2 * max(1, plan.splits) + 2 * M * N1 + 1024)
    gu.Workspace.ensure(need)
    dev = {k: gu.to_device(v, w.dtype) for k, v in host.items()}
    Y = torch.full((w.B, w.H, w.W, w.OC2), float("nan"), dtype=gu.torch_dtype(w.dtype), device="cuda")
    ff.ffuse_force_plan(plan)
    try:
        fn = ff.ffuse_conv_chain if w.dtype == "bf16" else ff.ffuse_conv_chain_f16
        fn(dev["X"], dev["W1"], dev["W2"], w.act, Y)
        ff.ffuse_sync_status()
        torch.cuda.synchronize()
    finally:
        ff.ffuse_force_plan(None)
    return Y


def check(Y, ref, dtype, what):
    got = gu.to_f64(Y)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    rel = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
    assert rel <= gu.TOL[dtype], f"{what}: relative error {rel:.3e}"
    return rel


@pytest.mark.parametrize("name", [f"C{i}" for i in range(1, 9)])
def test_paper_conv_chains(name):
    w = inputs.CONV_WORKLOADS[name]
    host = inputs.make_conv(w)
    ref = oracle.conv_chain(host["X"], host["W1"], host["W2"], w.act, bf16=True)
    print(name, "rel err", check(run_conv(w, host), ref, "bf16", name), flush=True)
    print(name, "again  ", check(run_conv(w, host), ref, "bf16", name + " again"), flush=True)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("act", [ACT_RELU, ACT_GELU_TANH, ACT_SILU])
def test_ragged_3x3_chains(dtype, act):
    cases = [(2, 5, 7, 64, 72, 40), (1, 1, 1, 64, 8, 8), (3, 9, 4, 128, 136, 264), (1, 13, 11, 192, 520, 24), (1, 1, 40, 64, 64, 64)]
    for i, (B, H, W, IC, OC1, OC2) in enumerate(cases):
        w = inputs.ConvWorkload(f"r{i}", B, H, W, IC, OC1, OC2, 3, 1, dtype, act, 400 + i)
        host = inputs.make_conv(w)
        ref = oracle.conv_chain(host["X"], host["W1"], host["W2"], act, bf16=(dtype == "bf16"))
        check(run_conv(w, host), ref, dtype, f"{dtype} {(B, H, W, IC, OC1, OC2)}")
        # row blocks and hidden slices of the 3x3 loader's kernels (slices of 128, 64 and 32 channels)
        for bm, bh, splits in ((32, 128, 2), (64, 128, 1), (128, 128, 3), (64, 64, 2), (128, 64, 1), (128, 32, 2)):
            if bm < 128 and B * H * W > bm:
                continue
            plan = ff.make_plan(ff.FAMILY_TWOPHASE, bm=bm, bh=bh, splits=splits, raster=2)
            check(run_conv(w, host, plan), ref, dtype, f"{dtype} {(B, H, W, IC, OC1, OC2)} bm={bm} bh={bh} splits={splits}")
            assert ff.ffuse_last_plan().bh == bh


def test_pointwise_chain_and_argument_errors():
    w = inputs.ConvWorkload("p", 2, 6, 5, 72, 136, 40, 1, 1, "bf16", ACT_RELU, 410)
    host = inputs.make_conv(w)
    ref = oracle.conv_chain(host["X"], host["W1"], host["W2"], w.act, bf16=True)
    check(run_conv(w, host), ref, "bf16", "1x1 chain")
    X = torch.zeros((1, 4, 4, 64), dtype=torch.bfloat16, device="cuda")
    Y = torch.zeros((1, 4, 4, 64), dtype=torch.bfloat16, device="cuda")
    W5 = torch.zeros((5, 5, 64, 64), dtype=torch.bfloat16, device="cuda")
    W3 = torch.zeros((3, 3, 64, 64), dtype=torch.bfloat16, device="cuda")
    W1 = torch.zeros((1, 1, 64, 64), dtype=torch.bfloat16, device="cuda")
    assert ff.ffuse_conv_chain(X, W5, W1, ACT_RELU, Y, check=False) == -2      # 5x5 first convolution
    assert ff.ffuse_conv_chain(X, W3, W3, ACT_RELU, Y, check=False) == -2      # 3x3 second convolution
    X40 = torch.zeros((1, 4, 4, 40), dtype=torch.bfloat16, device="cuda")
    W40 = torch.zeros((3, 3, 40, 64), dtype=torch.bfloat16, device="cuda")
    assert ff.ffuse_conv_chain(X40, W40, W1, ACT_RELU, Y, check=False) == -2   # 3x3 needs IC % 64 == 0
