"""CPU oracle (test infrastructure only): see expm_oracle.c for what it computes and how it is pinned."""
from .expm_oracle import (  # noqa: F401
    build_oracle,
    oracle_expm,
    oracle_expm_batch,
    oracle_matmul,
    oracle_max_threads,
    oracle_norm1,
    oracle_select,
    oracle_select_from_norms,
    oracle_b16,
    oracle_select_ps,
    oracle_select_ps_from_norms,
    oracle_expm_ps_batch,
    oracle_expm_baseline_batch,
    oracle_lowrank_batch,
    oracle_lowrank_select_from_norm,
)
