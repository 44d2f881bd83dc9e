"""Seeded synthetic inputs shared by the oracle tests, the GPU tests and bench.py.

This package holds no arithmetic of the SAMA method: only a counter-based
random generator, the recipes that turn it into data sets / initial
parameters / batches, and bit-level helpers (bf16 rounding of *inputs*).
"""
from .rng import CounterRNG, mix64
from .workloads import (WORKLOADS, Workload, make_workload, param_count,
                        param_layout, init_theta, init_lambda, init_lambda_corr, round_to_bf16,
                        flip_labels, make_aux_batch, make_aux_workload, AUX_TASK, seq_lengths)
