"""CPU oracle for the SlimAttention hot path.

TEST INFRASTRUCTURE ONLY.  Nothing under ``paper_2407_07304_amd/`` may import this
package; only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` do.  It shares no code with the HIP path.
"""
from .reference import (  # noqa: F401
    attn,
    attn_row_probs,
    attn_full_matrix_np,
    slim_attn_rowblocks_np,
    dequant_np,
    kv_quant_int8,
    kv_quant_int8_np,
    quant_division_sweep,
    num_threads,
    bf16_bits_to_f64,
)
from .build_oracle import build  # noqa: F401
