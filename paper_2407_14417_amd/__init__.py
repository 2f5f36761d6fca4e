"""Mixed-precision (16-bit / 4-bit experts) MoE feed-forward block for MI355X.

The compute lives in the HIP library ``libmoemix.so`` (sources under ``csrc/``,
C-ABI declared in ``include/moemix.h``); :mod:`paper_2407_14417_amd.binding`
marshals arguments to it and raises if the library is not built.
:mod:`paper_2407_14417_amd.synth` is the seeded input generator.
"""
__all__ = ["binding", "synth", "buildlib"]
