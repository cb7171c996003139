"""CPU oracle for the MAGE hot path -- test infrastructure only.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline``
leg may import this package.  It shares nothing with the HIP library.
"""
from .mage_oracle import (  # noqa: F401
    build,
    threads,
    block_probs,
    topk,
    select,
    exact_attn,
    sparse_attn,
    compact,
    page_summary,
    quest_probs,
    quest_select,
    overlap,
)
