"""Seeded synthetic inputs for the turn-resumption hot path.

This module only draws shapes, lengths, block tables and tensor values.  It holds none of the
arithmetic of pack, unpack or attention: both the CPU oracle's tests and the HIP path's tests /
benchmark take their inputs from here, and neither of those two imports the other.

Two kinds of values are produced:

* ``rng`` values: ``numpy.random.default_rng(seed)`` draws (N(0, sigma) for Q, K, V), rounded once
  to bf16 (round-to-nearest-even) on the host for the bf16 workloads.  Used wherever a tensor fits
  comfortably in host memory (attention inputs of one layer, all small test cases).
* ``counter`` values: a pure function of (seed, element index) built from 32-bit integer mixing,
  written so that numpy (host) and torch integer ops (device) produce identical bits.  Used to
  fill multi-layer K,V pools that are too large to generate on the host (pack / unpack only move
  bytes, so any bit pattern, NaN payloads included, is a valid input).
"""
from .configs import WorkloadConfig, CONFIGS, get_config, scaled_config
from .sessions import SessionBatch, UnitBatch, make_sessions, make_units
from .values import (
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    counter_bits_host,
    counter_bits_device,
    make_attn_inputs,
    make_attn_inputs_device,
    make_pool_host,
    fill_pool_blocks_device,
    SENTINEL16,
)

__all__ = [
    "WorkloadConfig", "CONFIGS", "get_config", "scaled_config",
    "SessionBatch", "UnitBatch", "make_sessions", "make_units",
    "f32_to_bf16_bits", "bf16_bits_to_f32", "counter_bits_host", "counter_bits_device",
    "make_attn_inputs", "make_attn_inputs_device", "make_pool_host", "fill_pool_blocks_device", "SENTINEL16",
]
