"""MoE-layer forward for AMD MI355X (gfx950): a C-ABI HIP library and its thin binding.

    from paper_2603_06350_amd import binding   # the five calls of include/moe.h
    from paper_2603_06350_amd import layer     # device buffers + the four-call forward
"""
from . import binding  # noqa: F401

__all__ = ["binding"]
