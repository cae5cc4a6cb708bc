"""Seeded synthetic workloads for the AMDP stage hot path.

This module serves both the CPU oracle's tests and the HIP library's tests and
benchmark. It holds configuration records and random-input recipes only: none
of the method's arithmetic (no transformer math, no optimizer, no schedule)
lives here, and it imports neither the oracle nor the HIP binding.
"""
from .configs import StageWorkload, CONFIGS, TINY, PAPER, FIRST, get
from .gen import (quantize_bf16_grid, make_theta, make_x, make_dy,
                  make_valid_len, make_targets, make_tokens, make_aux, stage_config_args, seed_for)

__all__ = ["StageWorkload", "CONFIGS", "TINY", "PAPER", "FIRST", "get", "quantize_bf16_grid",
           "make_theta", "make_x", "make_dy", "make_valid_len", "make_targets", "make_tokens",
           "make_aux", "stage_config_args", "seed_for"]
