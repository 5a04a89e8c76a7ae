"""fp64 CPU oracle for the fused FFN chain and the convolution chain -- TEST INFRASTRUCTURE ONLY.

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It is independent of the HIP library: no shared code, no import of
the product package, and no value in here ever comes from the GPU path.

The arithmetic lives in ``ffn_oracle.c`` (plain C loops in double, OpenMP over rows); this
module compiles it on demand with gcc and marshals numpy arrays into it.
"""
from .ffn_oracle import (  # noqa: F401
    ACT_IDENTITY,
    ACT_RELU,
    ACT_GELU_TANH,
    ACT_SILU,
    act,
    build,
    conv_chain,
    ffn,
    ffn_rows,
    num_threads,
    widen,
)
