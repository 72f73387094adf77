"""MI355X-native filter-gradient (weight-gradient) convolution, exact and in the
max-gradient approximation of arXiv 1908.05460.

The product is the C-ABI library built from ``csrc/`` (declared in
``include/wgrad.h``); ``binding`` marshals arguments into it and nothing else.
``inputs`` holds the seeded synthetic workloads, ``schedule`` the approximation
schedules (host-side masks).  Importing the package loads nothing native;
``binding.load()`` does, and raises if the HIP library has not been built.
"""
__all__ = ["binding", "inputs", "schedule", "build"]
