"""Helpers shared by the tests: host copies of synthetic models in the oracle's structs."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2511_00796_amd import synth


def host_model(shape, seed, n_layers=None):
    """(oracle.Weights, global dict, list of layer dicts) with uint16 bf16 bit patterns."""
    L = shape.n_layers if n_layers is None else n_layers
    g = {k: synth.as_u16(v) for k, v in synth.global_weights(shape, seed).items()}
    layers = [{k: synth.as_u16(v) for k, v in synth.layer_weights(shape, l, seed).items()} for l in range(L)]
    return oracle.Weights(g, layers), g, layers


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits_ref(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even bf16 by integer arithmetic on the fp32 pattern (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    low = u & 0xFFFF
    up = u >> 16
    inc = (low > 0x8000) | ((low == 0x8000) & ((up & 1) == 1))
    return (up + inc).astype(np.uint16)
