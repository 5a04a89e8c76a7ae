"""Seeded synthetic inputs for the FFN chains.  Holds NONE of the method's arithmetic.

This module serves both the HIP path's tests/bench and the CPU oracle's tests, so that both
sides consume bit-identical operand buffers.  It knows shapes, distributions and number
formats only.

Generator: counter-based.  Element ``i`` of the tensor with seed ``s`` is a pure function
of ``(s, i)``: two splitmix64 outputs -> two uniforms -> one Box-Muller normal (or one
uniform).  Values are produced in float64, scaled, rounded ONCE (round-to-nearest-even) to
the operand format, and returned as that format's storage array:

    "bf16" -> numpy.uint16 (upper half of the binary32 pattern)
    "f16"  -> numpy.float16
    "f32"  -> numpy.float32

Workloads (shapes are (M, K, N1, N2); paper notation (m, k, n, l), Evaluation, tables of
GEMM-chain and gated-FFN configurations):
  the five benchmark configurations, plus the paper's own m = 128 shape tables G1..G10
  (standard FFN) and S1..S8 (gated FFN).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

ACT_IDENTITY, ACT_RELU, ACT_GELU_TANH, ACT_SILU = 0, 1, 2, 3

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 16          # temporaries of one chunk stay cache-resident
_WORKERS = 16             # numpy releases the GIL inside its loops


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """One splitmix64 output per uint64 counter value (all arithmetic modulo 2^64)."""
    z = x + _GOLDEN
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _uniform01(bits: np.ndarray) -> np.ndarray:
    """53-bit uniform in (0, 1): never exactly 0 so that log() is finite."""
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _raw(seed: int, start: int, count: int, dist: str) -> np.ndarray:
    idx = np.arange(start, start + count, dtype=np.uint64)
    base = _splitmix64(np.full(1, seed, dtype=np.uint64))[0]
    with np.errstate(over="ignore"):
        c = idx * np.uint64(2) + base
        u1 = _uniform01(_splitmix64(c))
        if dist == "uniform":  # U(-1, 1)
            return 2.0 * u1 - 1.0
        u2 = _uniform01(_splitmix64(c + np.uint64(1)))
    if dist == "normal":  # N(0, 1), Box-Muller
        return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    raise ValueError(dist)


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float64/float32 -> bf16 bit patterns (uint16), round-to-nearest-even, finite inputs."""
    f = np.asarray(x, dtype=np.float32)  # float64 -> float32 is itself RNE; see note below
    u = f.view(np.uint32).astype(np.uint64)
    bias = np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))
    return ((u + bias) >> np.uint64(16)).astype(np.uint16)
# Note: the generator's float64 values pass through float32 before the bf16 rounding.  The
# stored buffer is what both sides consume, so a (vanishingly rare) double rounding changes
# nothing about parity: neither side ever sees the float64 value.


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def storage_dtype(dtype: str):
    return {"bf16": np.uint16, "f16": np.float16, "f32": np.float32}[dtype]


def tensor(seed: int, shape, dist: str, scale: float, dtype: str) -> np.ndarray:
    """Seeded tensor of ``shape``: ``scale * dist`` rounded once to ``dtype``."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=storage_dtype(dtype))

    def fill(s):
        c = min(_CHUNK, n - s)
        v = _raw(seed, s, c, dist) * scale
        if dtype == "bf16":
            out[s:s + c] = round_to_bf16_bits(v)
        elif dtype == "f16":
            out[s:s + c] = v.astype(np.float16)
        else:
            out[s:s + c] = v.astype(np.float32)

    starts = range(0, n, _CHUNK)
    if n > 8 * _CHUNK:
        workers = max(1, min(_WORKERS, os.cpu_count() or 1))
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fill, starts))
    else:
        for s in starts:
            fill(s)
    return out.reshape(shape)


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    K: int
    N1: int
    N2: int
    dtype: str       # "bf16" | "f16" | "f32"
    act: int
    gated: bool
    dist: str        # "normal" | "uniform"
    cfg_id: int      # seeds are 1000*cfg_id + tensor id (X=0, W1=1, W3=2, W2=3)

    @property
    def shape(self):
        return (self.M, self.K, self.N1, self.N2)

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2

    def flops(self) -> int:
        """Useful flops: 2*M*N1*(g*K + N2); activation arithmetic is not counted."""
        g = 2 if self.gated else 1
        return 2 * self.M * self.N1 * (g * self.K + self.N2)

    def q_min(self) -> int:
        """Compulsory bytes: X, the weights and Y, each moved once."""
        g = 2 if self.gated else 1
        e = self.elem_bytes
        return e * (self.M * self.K + g * self.K * self.N1 + self.N1 * self.N2 + self.M * self.N2)

    def q_unfused(self) -> int:
        """Compulsory bytes plus one write and one read of the intermediate."""
        return self.q_min() + 2 * self.elem_bytes * self.M * self.N1

    def with_m(self, m: int) -> "Workload":
        return Workload(f"{self.name}@m{m}", m, self.K, self.N1, self.N2, self.dtype, self.act,
                        self.gated, self.dist, self.cfg_id)


def _mk(name, M, K, N1, N2, dtype, act, gated, dist, cfg_id):
    return Workload(name, M, K, N1, N2, dtype, act, gated, dist, cfg_id)


# The five benchmark configurations.
WORKLOADS = {
    "tiny":     _mk("tiny", 128, 256, 1024, 256, "f32", ACT_RELU, False, "normal", 1),
    "gpt":      _mk("gpt", 4096, 4096, 16384, 4096, "bf16", ACT_GELU_TANH, False, "normal", 2),
    "llama":    _mk("llama", 2048, 4096, 11008, 4096, "bf16", ACT_SILU, True, "normal", 3),
    "decode16": _mk("decode16", 16, 8192, 28672, 8192, "bf16", ACT_SILU, True, "normal", 4),
    "decode64": _mk("decode64", 64, 8192, 28672, 8192, "bf16", ACT_SILU, True, "normal", 5),
    "large":    _mk("large", 32768, 1024, 8192, 1024, "f16", ACT_RELU, False, "uniform", 6),
}

# The paper's own shape tables (Evaluation: "configuration of gemm chain" / "gated FFN"),
# all at m = 128.  Paper order (m, n, k, l) -> ours (M, K, N1, N2) = (m, k, n, l).
_G = [(512, 32, 256), (256, 512, 64), (512, 416, 256), (3072, 768, 768), (16384, 4096, 4096),
      (4096, 1024, 1024), (768, 768, 768), (8192, 2048, 2048), (2048, 512, 512), (1536, 384, 384)]
_S = [(8192, 3072, 3072), (5632, 2048, 2048), (11008, 4096, 4096), (8192, 2048, 2048),
      (11008, 2048, 2048), (8960, 1536, 1536), (9728, 2560, 2560), (3072, 1024, 1024)]
for _i, (_n, _k, _l) in enumerate(_G):
    WORKLOADS[f"G{_i + 1}"] = _mk(f"G{_i + 1}", 128, _k, _n, _l, "bf16", ACT_GELU_TANH, False,
                                  "normal", 100 + _i)
for _i, (_n, _k, _l) in enumerate(_S):
    WORKLOADS[f"S{_i + 1}"] = _mk(f"S{_i + 1}", 128, _k, _n, _l, "bf16", ACT_SILU, True,
                                  "normal", 200 + _i)


@dataclass(frozen=True)
class ConvWorkload:
    """Two convolutions with an activation between them (paper: Evaluation, table "The
    configuration of conv chain"): channels-last image, stride 1, zero padding k/2."""
    name: str
    B: int
    H: int
    W: int
    IC: int
    OC1: int
    OC2: int
    k1: int
    k2: int
    dtype: str
    act: int
    cfg_id: int

    def gemm_shape(self):
        """(M, K, N1, N2) of the equivalent GEMM chain over pixel rows (k2 = 1)."""
        return (self.B * self.H * self.W, self.k1 * self.k1 * self.IC, self.OC1, self.OC2 * self.k2 * self.k2)

    def flops(self) -> int:
        npix = self.B * self.H * self.W
        return 2 * npix * self.OC1 * (self.k1 * self.k1 * self.IC + self.k2 * self.k2 * self.OC2)

    def q_min(self) -> int:
        npix = self.B * self.H * self.W
        return 2 * (npix * self.IC + self.k1 * self.k1 * self.IC * self.OC1 + self.k2 * self.k2 * self.OC1 * self.OC2 +
                    npix * self.OC2)


# The paper's conv-chain table (IC, H, W, OC1, OC2, k1, k2).  The table gives no batch size,
# activation or type: batch 1, ReLU between the convolutions and bf16 are this build's reading.
_C = [(64, 56, 56, 256, 64, 1, 1), (128, 28, 28, 512, 128, 1, 1), (256, 14, 14, 1024, 256, 1, 1),
      (512, 7, 7, 2048, 512, 1, 1), (64, 56, 56, 64, 256, 3, 1), (128, 28, 28, 128, 512, 3, 1),
      (256, 14, 14, 256, 1024, 3, 1), (512, 7, 7, 512, 2048, 3, 1)]
CONV_WORKLOADS = {
    f"C{_i + 1}": ConvWorkload(f"C{_i + 1}", 1, _h, _w, _ic, _o1, _o2, _k1, _k2, "bf16", ACT_RELU, 300 + _i)
    for _i, (_ic, _h, _w, _o1, _o2, _k1, _k2) in enumerate(_C)
}


def make_conv(w: ConvWorkload):
    """Operand buffers of a conv chain: X [B][H][W][IC] ~ N(0,1), W1 [k1][k1][IC][OC1] and
    W2 [k2][k2][OC1][OC2] ~ N(0, 1/fan_in) with fan_in = k*k*channels_in (storage arrays)."""
    s = 1000 * w.cfg_id
    X = tensor(s + 0, (w.B, w.H, w.W, w.IC), "normal", 1.0, w.dtype)
    W1 = tensor(s + 1, (w.k1, w.k1, w.IC, w.OC1), "normal", (w.k1 * w.k1 * w.IC) ** -0.5, w.dtype)
    W2 = tensor(s + 3, (w.k2, w.k2, w.OC1, w.OC2), "normal", (w.k2 * w.k2 * w.OC1) ** -0.5, w.dtype)
    return {"X": X, "W1": W1, "W2": W2}


def make(w: Workload, m_rows=None):
    """Operand buffers of a workload: dict with X, W1, W3 (or None), W2 (storage arrays).

    Distributions: "normal" -> X ~ N(0,1), W ~ N(0, 1/fan_in) (second argument a variance);
    "uniform" -> X ~ U(-1,1), W ~ U(-1,1)/sqrt(fan_in).  fan_in is K for W1/W3, N1 for W2.
    ``m_rows`` limits X to its first ``m_rows`` rows (same values as the full tensor's).
    """
    s = 1000 * w.cfg_id
    M = w.M if m_rows is None else min(w.M, m_rows)
    X = tensor(s + 0, (M, w.K), w.dist, 1.0, w.dtype)
    W1 = tensor(s + 1, (w.K, w.N1), w.dist, w.K ** -0.5, w.dtype)
    W3 = tensor(s + 2, (w.K, w.N1), w.dist, w.K ** -0.5, w.dtype) if w.gated else None
    W2 = tensor(s + 3, (w.N1, w.N2), w.dist, w.N1 ** -0.5, w.dtype)
    return {"X": X, "W1": W1, "W3": W3, "W2": W2}


def custom(name, M, K, N1, N2, dtype="bf16", act=ACT_RELU, gated=False, dist="normal", cfg_id=900):
    return _mk(name, M, K, N1, N2, dtype, act, gated, dist, cfg_id)


def sample_rows(M: int, block: int, per_block: int, seed: int) -> np.ndarray:
    """Stratified row sample: first and last row of every ``block``-row block plus
    ``per_block - 2`` seeded interior rows; sorted, unique."""
    rows = []
    nb = (M + block - 1) // block
    for b in range(nb):
        lo, hi = b * block, min(M, (b + 1) * block)
        rows += [lo, hi - 1]
        extra = max(0, per_block - 2)
        if extra and hi - lo > 2:
            r = _splitmix64(np.arange(extra, dtype=np.uint64) + np.uint64(seed * 7919 + b * 104729))
            rows += list(lo + (r % np.uint64(hi - lo)).astype(np.int64))
    return np.unique(np.asarray(rows, dtype=np.int64))
