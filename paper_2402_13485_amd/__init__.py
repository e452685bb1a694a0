"""MI355X-native token-tree verification (tree attention, early pruning, greedy acceptance).

The work is done by HIP kernels in ``libpropd.so`` (sources in ``csrc/``, C ABI in
``include/propd.h``).  ``binding`` marshals PyTorch device tensors into that ABI;
``synth`` generates seeded synthetic workloads; ``build`` compiles the library.
"""
from . import synth  # noqa: F401  (pure numpy, no GPU needed)

__all__ = ["synth", "binding", "build"]
