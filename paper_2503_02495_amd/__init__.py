"""MI355X-native forward pass of one Union-of-Experts layer (arXiv 2503.02495).

The product is the C-ABI library built from ``csrc/`` (declared in
``include/uoe.h``); ``binding`` marshals arguments to it and ``synth`` draws
seeded synthetic inputs.  Importing this package loads nothing native: the
library is opened on first use of ``binding`` and a missing build is an error.
"""
__all__ = ["synth", "binding", "build"]
