"""CPU checker (test infrastructure, not the product).

Plain float64 statement of what a pipeline stage computes (vit_oracle.c) and of
what stands before and after the encoder layers (surround.py), and of
the optimal partition by exhaustive enumeration plus an evaluation of the recurrence of the
paper's dynamic program (partition.py, partition_oracle.c).  Only tests, the
smoke check and the benchmark's CPU-baseline leg import this package; it
imports nothing from the GPU library.
"""
from .surround import embed_forward, head_forward, patches  # noqa: F401
from .vit import (OracleConfig, attention, gelu, layer_forward, layernorm, linear,  # noqa: F401
                  num_threads, round_bf16, stage_forward)
