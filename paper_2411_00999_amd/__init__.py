"""MI355X-native fused LayerNorm backward + per-example gradient norms + GNS estimator.

The compute lives in the C-ABI library built from ``csrc/`` (see ``include/lnpegn.h``);
``binding`` marshals arguments to it and ``workloads`` draws the seeded synthetic inputs.
Importing the package loads nothing; the library is loaded on first use and a missing
library is an error, never a fallback.
"""
__all__ = ["binding", "workloads", "build"]
