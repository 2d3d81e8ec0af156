"""CPU oracle of the frequency-aware embedding cache -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over fc_oracle.c (see that file's header for what it
defines and how it is pinned).  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library never does.
"""
from .wrapper import Oracle, OracleError, bag_sum, build  # noqa: F401
from .static_module import count_ids, freq_rank_from_counts, reorder_table  # noqa: F401
