"""CPU oracles for PCMM, for the ring-switch coefficient permutation and for the slot-encoded batch PCMM of
PC-attention, and for the ring products of the decode-time PCMv: test infrastructure only (see pcmm_oracle.c,
ring_switch_oracle.py, slot_pcmm_oracle.py and pcmv_oracle.c for what they compute).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
"""
from .pcmm_oracle import build_oracle, pcmm_oracle, pcmm_oracle_select, pcmm_freivalds, oracle_threads  # noqa: F401
from .ring_switch_oracle import ring_compose, ring_decompose  # noqa: F401
from . import slot_pcmm_oracle  # noqa: F401
from .pcmv_oracle import build_pcmv_oracle, pcmv_oracle, pcmv_oracle_rows  # noqa: F401
