"""MI355X-native hot path of SAR (sequential aggregation and rematerialization).

``paper_2111_06483_amd.sar`` is the thin binding over the C-ABI library built
from ``csrc/``; ``paper_2111_06483_amd.synth`` draws seeded synthetic inputs.
Importing the package loads neither torch kernels nor the shared library;
the binding loads the library on first use and raises if it is missing.
"""
__all__ = ["synth", "sar"]
