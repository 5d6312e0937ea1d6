"""SlimAttention prefill / INT8-KV decode for MI355X (gfx950).

``slimattn`` holds the bindings to the C-ABI library built from ``csrc/``; ``inputs``
the seeded workload generators; ``accounting`` the flop and byte counts.
"""
from . import accounting, inputs  # noqa: F401
