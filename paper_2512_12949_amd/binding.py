"""Thin ctypes binding of libffuse.so: same names as include/ffuse.h, argument marshalling
only.  Every step of the chain runs in the library's HIP kernels; there is no Python or
PyTorch fallback -- if the library is missing or the device is not gfx950 the calls raise.

PyTorch is used by callers for device memory and streams only: tensors are passed as
``data_ptr()`` values, streams as ``torch.cuda.current_stream().cuda_stream``.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libffuse.so")

ACT_IDENTITY, ACT_RELU, ACT_GELU_TANH, ACT_SILU = 0, 1, 2, 3
DT_BF16, DT_F16, DT_F32 = 0, 1, 2
FAMILY_AUTO, FAMILY_REDUCE, FAMILY_EXCHANGE, FAMILY_UNFUSED, FAMILY_SCALAR, FAMILY_TWOPHASE, FAMILY_ROWS = 0, 1, 2, 3, 4, 5, 6
DTYPE_CODE = {"bf16": DT_BF16, "f16": DT_F16, "f32": DT_F32}

EXPORTS = [
    "ffuse_ffn", "ffuse_ffn_f16", "ffuse_ffn_f32",
    "ffuse_ffn_unfused", "ffuse_ffn_unfused_f16", "ffuse_ffn_unfused_f32",
    "ffuse_workspace_bytes", "ffuse_set_workspace", "ffuse_choose_plan", "ffuse_traffic_model", "ffuse_plan_group_local",
    "ffuse_force_plan", "ffuse_last_plan", "ffuse_sync_status", "ffuse_profile_enable", "ffuse_profile_read",
    "ffuse_tune", "ffuse_plan_lookup", "ffuse_plan_table_clear", "ffuse_conv_chain", "ffuse_conv_chain_f16", "ffuse_rank_plans",
    "ffuse_plan_table_set", "ffuse_plan_table_save", "ffuse_plan_table_load",
    "ffuse_status_string", "ffuse_version",
    "ffuse_ffn_ws", "ffuse_ffn_unfused_ws", "ffuse_debug_barrier", "ffuse_set_objective",
    "ffuse_loop_schedule_count", "ffuse_cluster_exchange", "ffuse_ffn_static", "ffuse_calibrate",
]


class Plan(ctypes.Structure):
    _fields_ = [("family", ctypes.c_int32), ("bm", ctypes.c_int32), ("bh", ctypes.c_int32),
                ("bn2", ctypes.c_int32), ("bk", ctypes.c_int32), ("splits", ctypes.c_int32),
                ("h_level", ctypes.c_int32), ("raster", ctypes.c_int32), ("producers", ctypes.c_int32),
                ("ring", ctypes.c_int32), ("coherent", ctypes.c_int32), ("gate_split", ctypes.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class Traffic(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in (
        "flops", "hbm_bytes", "fabric_bytes", "l2_bytes", "lds_bytes", "reduce_bytes", "exchange_bytes",
        "q_min", "q_unfused", "t_mfma", "t_hbm", "t_fabric", "t_l2", "t_lds", "t_reduce", "t_pred",
        "lds_used", "acc_regs")] + [("feasible", ctypes.c_int32), ("workgroups", ctypes.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class FfuseError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: status {code} ({status_string(code)})")
        self.code = code


_lib = None


def lib():
    """Loads libffuse.so (built by ``paper_2512_12949_amd.build``); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: run `python -m paper_2512_12949_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        for name in EXPORTS[:6]:
            f = getattr(L, name)
            f.restype = ci
            f.argtypes = [vp, vp, vp, vp, ci, i64, i64, i64, i64, vp, vp]
        L.ffuse_workspace_bytes.restype = ctypes.c_size_t
        L.ffuse_workspace_bytes.argtypes = [ci, ci, i64, i64, i64, i64, ci]
        L.ffuse_set_workspace.restype = ci
        L.ffuse_set_workspace.argtypes = [vp, ctypes.c_size_t, vp]
        L.ffuse_choose_plan.restype = ci
        L.ffuse_choose_plan.argtypes = [ci, ci, ci, i64, i64, i64, i64, ctypes.POINTER(Plan)]
        L.ffuse_plan_group_local.restype = ci
        L.ffuse_plan_group_local.argtypes = [ctypes.POINTER(Plan), ci, ci, i64, i64, i64, i64]
        L.ffuse_traffic_model.restype = ci
        L.ffuse_traffic_model.argtypes = [ctypes.POINTER(Plan), ci, ci, i64, i64, i64, i64, ctypes.POINTER(Traffic)]
        L.ffuse_force_plan.restype = ci
        L.ffuse_force_plan.argtypes = [ctypes.POINTER(Plan)]
        L.ffuse_last_plan.restype = ci
        L.ffuse_last_plan.argtypes = [ctypes.POINTER(Plan)]
        L.ffuse_sync_status.restype = ci
        L.ffuse_sync_status.argtypes = [vp]
        L.ffuse_profile_enable.restype = ci
        L.ffuse_profile_enable.argtypes = [ci]
        L.ffuse_profile_read.restype = ci
        L.ffuse_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        L.ffuse_tune.restype = ci
        L.ffuse_tune.argtypes = [ci, vp, vp, vp, vp, ci, i64, i64, i64, i64, vp, ci, ci, vp, ctypes.POINTER(Plan),
                                 ctypes.POINTER(ctypes.c_double)]
        L.ffuse_plan_lookup.restype = ci
        L.ffuse_plan_lookup.argtypes = [ci, ci, ci, i64, i64, i64, i64, ctypes.POINTER(Plan), ctypes.POINTER(ctypes.c_double)]
        L.ffuse_plan_table_clear.restype = ci
        L.ffuse_rank_plans.restype = ci
        L.ffuse_plan_table_set.restype = ci
        L.ffuse_plan_table_set.argtypes = [ci, ci, i64, i64, i64, i64, ctypes.POINTER(Plan), ctypes.c_double]
        L.ffuse_plan_table_save.restype = ci
        L.ffuse_plan_table_save.argtypes = [ctypes.c_char_p]
        L.ffuse_plan_table_load.restype = ci
        L.ffuse_plan_table_load.argtypes = [ctypes.c_char_p]
        L.ffuse_rank_plans.argtypes = [ci, ci, ci, i64, i64, i64, i64, ctypes.POINTER(Plan), ctypes.POINTER(ctypes.c_double), ci]
        for name in ("ffuse_conv_chain", "ffuse_conv_chain_f16"):
            f = getattr(L, name)
            f.restype = ci
            f.argtypes = [vp, vp, vp, ci, i64, i64, i64, i64, i64, i64, ci, ci, vp, vp]
        L.ffuse_status_string.restype = ctypes.c_char_p
        L.ffuse_status_string.argtypes = [ci]
        L.ffuse_version.restype = ci
        for name in ("ffuse_ffn_ws", "ffuse_ffn_unfused_ws"):
            f = getattr(L, name)
            f.restype = ci
            f.argtypes = [ci, vp, vp, vp, vp, ci, i64, i64, i64, i64, vp, vp, ctypes.c_size_t, vp]
        L.ffuse_loop_schedule_count.restype = ci
        L.ffuse_loop_schedule_count.argtypes = [ci]
        L.ffuse_cluster_exchange.restype = ci
        L.ffuse_cluster_exchange.argtypes = [ci, ci, ci, ctypes.POINTER(ci), ctypes.POINTER(ci)]
        L.ffuse_set_objective.restype = ci
        L.ffuse_set_objective.argtypes = [ci]
        L.ffuse_ffn_static.restype = ci
        L.ffuse_ffn_static.argtypes = [ci, vp, vp, vp, vp, ci, i64, i64, i64, i64, vp, vp]
        L.ffuse_calibrate.restype = ci
        L.ffuse_calibrate.argtypes = [ci, ci, vp, i64, i64, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.ffuse_debug_barrier.restype = ci
        L.ffuse_debug_barrier.argtypes = [ci, ctypes.c_uint]
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().ffuse_status_string(int(code)).decode()


def _check(code, what):
    if code != 0:
        raise FfuseError(code, what)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(int(t.data_ptr()) if hasattr(t, "data_ptr") else int(t))


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(int(stream))


def _call(name, X, W1, W3, W2, act, Y, stream, check):
    M, K = X.shape
    N1, N2 = W2.shape
    rc = getattr(lib(), name)(_ptr(X), _ptr(W1), _ptr(W3), _ptr(W2), int(act), M, K, N1, N2, _ptr(Y), _stream(stream))
    if check:
        _check(rc, name)
    return rc


def ffuse_ffn(X, W1, W3, W2, act, Y, stream=None, check=True):
    return _call("ffuse_ffn", X, W1, W3, W2, act, Y, stream, check)


def ffuse_ffn_f16(X, W1, W3, W2, act, Y, stream=None, check=True):
    return _call("ffuse_ffn_f16", X, W1, W3, W2, act, Y, stream, check)


def ffuse_ffn_f32(X, W1, W3, W2, act, Y, stream=None, check=True):
    return _call("ffuse_ffn_f32", X, W1, W3, W2, act, Y, stream, check)


def ffuse_ffn_unfused(X, W1, W3, W2, act, Y, stream=None, check=True):
    return _call("ffuse_ffn_unfused", X, W1, W3, W2, act, Y, stream, check)


def ffuse_ffn_unfused_f16(X, W1, W3, W2, act, Y, stream=None, check=True):
    return _call("ffuse_ffn_unfused_f16", X, W1, W3, W2, act, Y, stream, check)


def ffuse_ffn_unfused_f32(X, W1, W3, W2, act, Y, stream=None, check=True):
    return _call("ffuse_ffn_unfused_f32", X, W1, W3, W2, act, Y, stream, check)


def _call_ws(name, dtype, X, W1, W3, W2, act, Y, workspace, stream, check):
    M, K = X.shape
    N1, N2 = W2.shape
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = getattr(lib(), name)(int(dtype), _ptr(X), _ptr(W1), _ptr(W3), _ptr(W2), int(act), M, K, N1, N2, _ptr(Y),
                              _ptr(workspace), nbytes, _stream(stream))
    if check:
        _check(rc, name)
    return rc


def ffuse_ffn_ws(dtype, X, W1, W3, W2, act, Y, workspace, stream=None, check=True):
    """The fused chain with the workspace named per call (``workspace``: a device tensor, or None)."""
    return _call_ws("ffuse_ffn_ws", dtype, X, W1, W3, W2, act, Y, workspace, stream, check)


def ffuse_ffn_unfused_ws(dtype, X, W1, W3, W2, act, Y, workspace, stream=None, check=True):
    return _call_ws("ffuse_ffn_unfused_ws", dtype, X, W1, W3, W2, act, Y, workspace, stream, check)


def ffuse_loop_schedule_count(spatial_dims=0) -> int:
    return int(lib().ffuse_loop_schedule_count(int(spatial_dims)))


def ffuse_cluster_exchange(cls_n, cls_k, cls_l):
    """Returns (cls_shuffle, cls_reduce)."""
    a, b = ctypes.c_int(), ctypes.c_int()
    _check(lib().ffuse_cluster_exchange(int(cls_n), int(cls_k), int(cls_l), ctypes.byref(a), ctypes.byref(b)), "ffuse_cluster_exchange")
    return a.value, b.value


OBJECTIVE_TIME, OBJECTIVE_BYTES = 0, 1


def ffuse_set_objective(objective):
    _check(lib().ffuse_set_objective(int(objective)), "ffuse_set_objective")


def ffuse_ffn_static(dtype, X, W1, W3, W2, act, Y, stream=None, check=True):
    """The fused chain in the library's built-in 32 MiB of scratch memory: nothing is allocated."""
    M, K = X.shape
    N1, N2 = W2.shape
    rc = lib().ffuse_ffn_static(int(dtype), _ptr(X), _ptr(W1), _ptr(W3), _ptr(W2), int(act), M, K, N1, N2, _ptr(Y), _stream(stream))
    if check:
        _check(rc, "ffuse_ffn_static")
    return rc


CAL_MFMA, CAL_READ, CAL_MFMA_IDLE = 0, 1, 2


def ffuse_calibrate(what, dtype=DT_BF16, buf=None, iters=1, scratch=None, stream=None):
    """flop/s of the bare matrix-core issue loop (CAL_MFMA) or bytes/s of a streaming read of `buf` (CAL_READ)."""
    out = ctypes.c_double(0.0)
    nbytes = 0 if buf is None else buf.numel() * buf.element_size()
    _check(lib().ffuse_calibrate(int(what), int(dtype), _ptr(buf), nbytes, int(iters), _ptr(scratch), ctypes.byref(out), _stream(stream)),
           "ffuse_calibrate")
    return out.value


def ffuse_debug_barrier(extra_arrivals=0, spin_limit=1 << 24):
    _check(lib().ffuse_debug_barrier(int(extra_arrivals), int(spin_limit)), "ffuse_debug_barrier")


FUSED = {"bf16": ffuse_ffn, "f16": ffuse_ffn_f16, "f32": ffuse_ffn_f32}
UNFUSED = {"bf16": ffuse_ffn_unfused, "f16": ffuse_ffn_unfused_f16, "f32": ffuse_ffn_unfused_f32}


def ffuse_workspace_bytes(dtype, gated, M, K, N1, N2, unfused=False) -> int:
    return int(lib().ffuse_workspace_bytes(int(dtype), int(bool(gated)), M, K, N1, N2, int(bool(unfused))))


def ffuse_set_workspace(buf, nbytes=None, stream=None):
    if buf is None:
        _check(lib().ffuse_set_workspace(None, 0, _stream(stream)), "ffuse_set_workspace")
        return
    if nbytes is None:
        nbytes = buf.numel() * buf.element_size()
    _check(lib().ffuse_set_workspace(_ptr(buf), int(nbytes), _stream(stream)), "ffuse_set_workspace")


def ffuse_choose_plan(dtype, act, gated, M, K, N1, N2) -> Plan:
    p = Plan()
    _check(lib().ffuse_choose_plan(int(dtype), int(act), int(bool(gated)), M, K, N1, N2, ctypes.byref(p)),
           "ffuse_choose_plan")
    return p


def ffuse_plan_group_local(plan: Plan, dtype, gated, M, K, N1, N2) -> bool:
    rc = lib().ffuse_plan_group_local(ctypes.byref(plan), int(dtype), int(bool(gated)), M, K, N1, N2)
    if rc < 0:
        _check(rc, "ffuse_plan_group_local")
    return bool(rc)


def ffuse_traffic_model(plan: Plan, dtype, gated, M, K, N1, N2) -> Traffic:
    t = Traffic()
    _check(lib().ffuse_traffic_model(ctypes.byref(plan), int(dtype), int(bool(gated)), M, K, N1, N2, ctypes.byref(t)),
           "ffuse_traffic_model")
    return t


def ffuse_force_plan(plan):
    _check(lib().ffuse_force_plan(None if plan is None else ctypes.byref(plan)), "ffuse_force_plan")


def ffuse_last_plan() -> Plan:
    p = Plan()
    _check(lib().ffuse_last_plan(ctypes.byref(p)), "ffuse_last_plan")
    return p


def ffuse_sync_status(stream=None, check=True):
    rc = lib().ffuse_sync_status(_stream(stream))
    if check:
        _check(rc, "ffuse_sync_status")
    return rc


def ffuse_tune(dtype, X, W1, W3, W2, act, Y, top_k=6, reps=5, stream=None):
    """Returns (plan, milliseconds) of the fastest of the top_k modelled plans, now in the plan table."""
    M, K = X.shape
    N1, N2 = W2.shape
    p, ms = Plan(), ctypes.c_double()
    _check(lib().ffuse_tune(int(dtype), _ptr(X), _ptr(W1), _ptr(W3), _ptr(W2), int(act), M, K, N1, N2, _ptr(Y),
                            int(top_k), int(reps), _stream(stream), ctypes.byref(p), ctypes.byref(ms)), "ffuse_tune")
    return p, ms.value


def ffuse_plan_lookup(dtype, act, gated, M, K, N1, N2):
    """Returns (plan, tuned_ms): the plan a fused call would use now; tuned_ms is 0 for a modelled plan."""
    p, ms = Plan(), ctypes.c_double()
    _check(lib().ffuse_plan_lookup(int(dtype), int(act), int(bool(gated)), M, K, N1, N2, ctypes.byref(p), ctypes.byref(ms)),
           "ffuse_plan_lookup")
    return p, ms.value


def ffuse_rank_plans(dtype, act, gated, M, K, N1, N2, capacity=256):
    """The model's ranking: list of (plan, predicted seconds), best first."""
    plans = (Plan * capacity)()
    t = (ctypes.c_double * capacity)()
    n = lib().ffuse_rank_plans(int(dtype), int(act), int(bool(gated)), M, K, N1, N2, plans, t, capacity)
    if n < 0:
        raise FfuseError(n, "ffuse_rank_plans")
    out = []
    for i in range(n):
        p = Plan()
        ctypes.memmove(ctypes.byref(p), ctypes.byref(plans[i]), ctypes.sizeof(Plan))
        out.append((p, t[i]))
    return out


def ffuse_plan_table_set(dtype, gated, M, K, N1, N2, plan: Plan, ms=1.0):
    _check(lib().ffuse_plan_table_set(int(dtype), int(bool(gated)), M, K, N1, N2, ctypes.byref(plan), float(ms)),
           "ffuse_plan_table_set")


def ffuse_plan_table_save(path) -> int:
    n = lib().ffuse_plan_table_save(os.fsencode(path))
    if n < 0:
        raise FfuseError(n, "ffuse_plan_table_save")
    return n


def ffuse_plan_table_load(path) -> int:
    n = lib().ffuse_plan_table_load(os.fsencode(path))
    if n < 0:
        raise FfuseError(n, "ffuse_plan_table_load")
    return n


SHIPPED_PLANS = os.path.join(HERE, "plans_mi355x.txt")


def ffuse_load_shipped_plans() -> int:
    """Loads the plan table measured on an MI355X for the benchmark configurations and the paper's m = 128
    shapes (written by ``python -m paper_2512_12949_amd.tune_plans``); returns the number of entries, 0 if
    the file is not there.  Fused calls on those shapes (same dtype, gate, K, N1, N2, same bin of M) then
    use the measured plan instead of the model's choice."""
    return ffuse_plan_table_load(SHIPPED_PLANS) if os.path.exists(SHIPPED_PLANS) else 0


def ffuse_plan_table_clear():
    _check(lib().ffuse_plan_table_clear(), "ffuse_plan_table_clear")


def _conv(name, X, W1, W2, act, Y, stream, check):
    B, H, W, IC = X.shape
    k1, _, _, OC1 = W1.shape
    k2, _, _, OC2 = W2.shape
    rc = getattr(lib(), name)(_ptr(X), _ptr(W1), _ptr(W2), int(act), B, H, W, IC, OC1, OC2, k1, k2, _ptr(Y), _stream(stream))
    if check:
        _check(rc, name)
    return rc


def ffuse_conv_chain(X, W1, W2, act, Y, stream=None, check=True):
    """X [B][H][W][IC], W1 [k1][k1][IC][OC1], W2 [k2][k2][OC1][OC2], Y [B][H][W][OC2] (bf16)."""
    return _conv("ffuse_conv_chain", X, W1, W2, act, Y, stream, check)


def ffuse_conv_chain_f16(X, W1, W2, act, Y, stream=None, check=True):
    return _conv("ffuse_conv_chain_f16", X, W1, W2, act, Y, stream, check)


def ffuse_profile_enable(on: bool):
    _check(lib().ffuse_profile_enable(int(bool(on))), "ffuse_profile_enable")


def ffuse_profile_read():
    ms, n = ctypes.c_double(), ctypes.c_int64()
    _check(lib().ffuse_profile_read(ctypes.byref(ms), ctypes.byref(n)), "ffuse_profile_read")
    return ms.value, n.value


def ffuse_version() -> int:
    return int(lib().ffuse_version())


def make_plan(family, bm=0, bh=0, bn2=128, bk=64, splits=0, h_level=0, raster=4, producers=0, ring=0, coherent=0, gate_split=0) -> Plan:
    p = Plan()
    p.family, p.bm, p.bh, p.bn2, p.bk, p.splits, p.h_level, p.raster = family, bm, bh, bn2, bk, splits, h_level, raster
    p.producers, p.ring, p.coherent, p.gate_split = producers, ring, coherent, gate_split
    return p
