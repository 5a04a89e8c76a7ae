"""Helpers for the GPU parity tests: upload seeded operands, run the HIP path through the
C ABI, bring results back as float64, compare with the CPU oracle."""
import numpy as np
import torch

import oracle
from paper_2512_12949_amd import binding as ff
from paper_2512_12949_amd import inputs

# Tolerances of the parity bar: max|Y - Y_ref| <= tol * max|Y_ref|.
TOL = {"bf16": 2e-2, "f16": 2e-2, "f32": 1e-3}


def to_device(a, dtype):
    if a is None:
        return None
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def torch_dtype(dtype):
    return {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dtype]


class Workspace:
    """One caller-owned workspace, grown on demand and registered with the library."""
    buf = None

    @classmethod
    def ensure(cls, nbytes):
        nbytes = max(256, (nbytes + 255) // 256 * 256)
        if cls.buf is None or cls.buf.numel() < nbytes:
            cls.buf = None
            ff.ffuse_set_workspace(None)
            cls.buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            ff.ffuse_set_workspace(cls.buf)
            torch.cuda.synchronize()


def run(w, dev, unfused=False, plan=None):
    """Runs one workload on device tensors ``dev``; returns Y as a device tensor."""
    M = dev["X"].shape[0]
    dt = ff.DTYPE_CODE[w.dtype]
    need = max(ff.ffuse_workspace_bytes(dt, w.gated, M, w.K, w.N1, w.N2, False),
               ff.ffuse_workspace_bytes(dt, w.gated, M, w.K, w.N1, w.N2, True))
    if plan is not None and plan.family == ff.FAMILY_TWOPHASE:
        # a forced plan may ask for more partial planes than the chooser would ever use
        need = max(need, 4 * M * w.N2 * max(1, plan.splits) + (1 + plan.gate_split) * (2 * M * w.N1 + 256) + 1024)
    Workspace.ensure(need)
    Y = torch.full((M, w.N2), float("nan"), dtype=torch_dtype(w.dtype), device="cuda")
    ff.ffuse_force_plan(plan)
    try:
        fn = (ff.UNFUSED if unfused else ff.FUSED)[w.dtype]
        fn(dev["X"], dev["W1"], dev["W3"], dev["W2"], w.act, Y)
        ff.ffuse_sync_status()
        torch.cuda.synchronize()
    finally:
        ff.ffuse_force_plan(None)
    return Y


def oracle_rows(w, host, rows=None):
    return oracle.ffn_rows(host["X"], host["W1"], host["W3"], host["W2"], w.act, rows=rows, bf16=(w.dtype == "bf16"))


def check(Y, ref, dtype, rows=None, what=""):
    got = to_f64(Y if rows is None else Y[torch.as_tensor(np.asarray(rows), device=Y.device)])
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    scale = np.max(np.abs(ref))
    err = np.max(np.abs(got - ref)) if got.size else 0.0
    if scale == 0.0:
        assert err == 0.0, f"{what}: expected exact zeros"
        return 0.0
    rel = err / scale
    assert rel <= TOL[dtype], f"{what}: max|Y-Yref| = {rel:.3e} * max|Yref| exceeds {TOL[dtype]}"
    return rel
