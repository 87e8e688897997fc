"""MI355X-native decode hot path of TokenButler (arXiv 2503.07518): HIP kernels for gfx950 behind
a C ABI (``include/tokenbutler.h``), with this thin ctypes binding on top.

    from paper_2503_07518_amd import binding as tb
    tb.tb_score(desc, q_imp, Kimp, 1.0, scores)

``workloads`` holds the seeded synthetic input generators (no method arithmetic).
The HIP library is loaded on first use and its absence is an error: there is no CPU fallback.
"""
from . import binding, workloads  # noqa: F401

__all__ = ["binding", "workloads"]
