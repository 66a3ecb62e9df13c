"""Seeded synthetic input generators shared by the oracle's and the HIP library's tests."""
from .gen import (BASE_SEED, HEAD_MAJOR, TOKEN_MAJOR, VerifyBatch, arena_view, bits, from_bits,
                  make_batch, make_config, grow_trees, draw_lengths, strides_for, CONFIG_NAMES,
                  PaddedBatch, pad_batch, LoopStep, VerifyLoop, make_verify_loop)

__all__ = ["BASE_SEED", "HEAD_MAJOR", "TOKEN_MAJOR", "VerifyBatch", "arena_view", "bits",
           "from_bits", "make_batch", "grow_trees", "PaddedBatch", "pad_batch", "LoopStep", "VerifyLoop", "make_verify_loop", "make_config", "draw_lengths", "strides_for", "CONFIG_NAMES"]
