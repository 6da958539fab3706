"""Materialises a synthetic workload on the GPU through the C ABI: packs seeded random weights,
fills the paged cache with seeded K/V layer by layer (so that neither the 14-28 GB of weights nor
the 64-110 GB of cache ever sit on the host), and returns the device-side step inputs.

Pure orchestration of ``synth`` (inputs) and ``binding`` (the library); an optional ``tap`` callback
sees each layer's tensors as they are produced, which the tests use to hand the same inputs to the
CPU checker.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Callable, Optional

import numpy as np
import torch

from . import binding, synth


@dataclass
class DeviceWorkload:
    wl: synth.Workload
    engine: "binding.Engine"
    kv: "binding.KVCache"
    ctx: np.ndarray            # tokens cached before the step, per sequence
    seq_lens: np.ndarray       # keys attended in the step = ctx + 1
    table: np.ndarray          # [batch, max_blocks] host copy
    seq_start: np.ndarray      # [batch + 1] offsets of the cached tokens
    tokens_h: np.ndarray
    tokens: torch.Tensor
    positions: torch.Tensor
    seq_lens_d: torch.Tensor
    table_d: torch.Tensor
    logits: torch.Tensor
    next_tokens: torch.Tensor

    def step(self, with_logits: bool = True) -> None:
        self.engine.decode_step(self.kv, self.tokens, self.positions, self.seq_lens_d, self.table_d,
                                self.logits if with_logits else None, self.next_tokens)

    def bytes(self):
        return synth.algorithmic_bytes(self.wl.shape, self.seq_lens,
                                       1 if self.engine.cfg.kv_dtype == binding.HX_KV_FP8_E4M3 else 2)


def build(wl: synth.Workload, device="cuda:0", n_layers: Optional[int] = None,
          tap: Optional[Callable[[str, int, dict], None]] = None, max_seq_len: Optional[int] = None,
          kv_dtype: int = binding.HX_KV_BF16) -> DeviceWorkload:
    """Build the engine and a cache pre-filled with N(0,1) K/V for ``wl`` (kv_fill == "normal").

    ``n_layers`` truncates the model (parity tests on mid-size cases).  ``tap(kind, layer, tensors)``
    is called with kind "layer" (weights dict), "kv" ({"k", "v"} of that layer, logical layout) and
    "globals" (first) while the device tensors are alive.  ``kv_dtype``: element type of the cache (the bf16
    K/V handed to prefill_fill are rounded to it by the library).
    """
    shape = wl.shape
    if n_layers is not None:
        shape = dataclasses.replace(shape, n_layers=n_layers)
        wl = dataclasses.replace(wl, shape=shape)
    dev = torch.device(device)
    ctx = synth.context_lengths(wl)
    seq_lens = (ctx + 1).astype(np.int32)
    table, num_blocks = synth.block_table(seq_lens, shape.block_size, wl.seed)
    seq_start = np.concatenate([[0], np.cumsum(ctx)]).astype(np.int32)
    total = int(ctx.sum())
    msl = int(seq_lens.max()) if max_seq_len is None else max_seq_len
    eng = binding.Engine(shape, wl.batch, msl, device=device, kv_dtype=kv_dtype)
    kv = binding.KVCache(eng, num_blocks)
    table_d = torch.from_numpy(table).to(dev)
    start_d = torch.from_numpy(seq_start).to(dev)
    g = synth.global_weights(shape, wl.seed, device=dev)
    eng.pack_globals(g)
    if tap:
        tap("globals", 0, g)
    torch.cuda.synchronize(dev)
    del g
    for l in range(shape.n_layers):
        w = synth.layer_weights(shape, l, wl.seed, device=dev)
        eng.pack_layer(l, w)
        if tap:
            tap("layer", l, w)
        del w
        if wl.kv_fill == "normal" and total > 0:
            k, v = synth.kv_fill(shape, l, total, wl.seed, device=dev)
            kv.prefill_fill(l, k, v, start_d, table_d)
            if tap:
                tap("kv", l, {"k": k, "v": v})
            torch.cuda.synchronize(dev)
            del k, v
    torch.cuda.synchronize(dev)
    tokens_h = synth.token_ids(wl, wl.batch)
    return DeviceWorkload(
        wl=wl, engine=eng, kv=kv, ctx=ctx, seq_lens=seq_lens, table=table, seq_start=seq_start, tokens_h=tokens_h,
        tokens=torch.from_numpy(tokens_h).to(dev), positions=torch.from_numpy(ctx.astype(np.int32)).to(dev),
        seq_lens_d=torch.from_numpy(seq_lens).to(dev), table_d=table_d,
        logits=torch.empty(wl.batch, shape.vocab, dtype=torch.float32, device=dev),
        next_tokens=torch.empty(wl.batch, dtype=torch.int32, device=dev))
