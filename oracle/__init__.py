"""CPU oracles for PCMM and for the ring-switch coefficient permutation: test infrastructure only
(see pcmm_oracle.c and ring_switch_oracle.py for what they compute).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
"""
from .pcmm_oracle import build_oracle, pcmm_oracle, pcmm_oracle_select, pcmm_freivalds, oracle_threads  # noqa: F401
from .ring_switch_oracle import ring_compose, ring_decompose  # noqa: F401
