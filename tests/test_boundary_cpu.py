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
        return (r(4 * M * N2 * planes) if planes > 1 else 0) + r(2 * M * N1) + 256
    ring = 8192 + 8 * 64 * 256 * 256 * 2
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 4096, 4096, 16384, 4096, False) == max(4 * 4096 * 4096, ring, two_phase(4096, 16384, 4096, 1))
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 32768, 1024, 8192, 1024, False) == max(4 * 32768 * 1024, two_phase(32768, 8192, 1024, 1))
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 8192, 1024, 8192, 1024, False) == max(4 * 8192 * 1024, ring, two_phase(8192, 8192, 1024, 2))
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, True, 64, 64, 64, 64, False) == max(8192 + 8 * 64 * 256 * 128 * 2, two_phase(64, 64, 64, 32))
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 512, 4096, 16384, 4096, False) == max(ring, two_phase(512, 16384, 4096, 8))
    assert ff.ffuse_workspace_bytes(ff.DT_BF16, False, 4096, 4096, 16384, 4096, True) == 2 * 4096 * 16384
    assert ff.ffuse_workspace_bytes(ff.DT_F32, False, 128, 256, 1024, 256, True) == 4 * 128 * 1024
    assert ff.ffuse_workspace_bytes(ff.DT_F32, False, 128, 256, 1024, 256, False) == 0
