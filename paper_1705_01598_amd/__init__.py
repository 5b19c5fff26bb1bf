"""MI355X-native rank-n tensor transpose (plan + execute) behind a C-ABI library.

``paper_1705_01598_amd.binding`` wraps the shared library ``libtperm.so`` built from
``csrc/``; ``paper_1705_01598_amd.workloads`` holds the seeded synthetic shapes.  The
library is loaded on first use so that shape generation works without it; every
compute call fails loudly if it is missing.
"""

__all__ = ["binding", "workloads"]
