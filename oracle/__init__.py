"""CPU oracle for PCMM: test infrastructure only (see pcmm_oracle.c for what it computes).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
"""
from .pcmm_oracle import build_oracle, pcmm_oracle, pcmm_oracle_select, pcmm_freivalds, oracle_threads  # noqa: F401
