"""CPU oracle (test infrastructure only; never imported by the product path)."""
from .oracle import (attn_probe, attn_probe_batch, steer, steer_batch, residual_steer, round_bf16, num_threads,
                     build_oracle, lib_path, fp8_e4m3_value)

__all__ = ["attn_probe", "attn_probe_batch", "steer", "steer_batch", "residual_steer", "round_bf16", "num_threads",
           "build_oracle", "lib_path", "fp8_e4m3_value"]
