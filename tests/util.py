"""Helpers shared by the tests: host copies of synthetic models in the oracle's structs."""
from __future__ import annotations

import os

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


class OracleRows:
    """Runs the CPU oracle for a few sampled rows of a large workload, layer by layer, as the
    workload builder produces each layer's tensors on the GPU (`tap` protocol of
    paper_2511_00796_amd.workload.build).  Rows are independent in the decode step, so the sampled
    rows' results are exactly what the full-batch oracle would give for them."""

    def __init__(self, shape, rows, ctx, seq_start, tokens, descending=False, kv_fp8=False, keep_layers=()):
        from concurrent.futures import ThreadPoolExecutor
        self.shape, self.rows = shape, list(rows)
        self.descending = descending          # run the equally valid variant of the oracle with every sum reversed
        self.keep_layers = set(keep_layers)   # layers whose residual stream before / after, intermediate results and
        self.x_before, self.x_after = {}, {}  # product magnitudes sum_k |x_k w_kn| are kept per row
        self.trace, self.mag, self.layer_bias = {}, {}, {}
        self.ctx, self.seq_start, self.tokens = ctx, seq_start, tokens
        self.cfg1 = oracle.make_config(shape, kv_fp8=kv_fp8)   # kv_fp8: the 8-bit cache variant
        self.cfg1.n_layers = 1
        self.pool = ThreadPoolExecutor(max_workers=min(len(self.rows), 16))
        self.x = {}
        self.attn = {r: [] for r in self.rows}
        self.globals = None
        self.layer_w = None
        self.logits, self.next = {}, {}

    def tap(self, kind, layer, t):
        if self.descending:
            with oracle.descending_sums():
                return self._tap(kind, layer, t)
        return self._tap(kind, layer, t)

    def _tap(self, kind, layer, t):
        if kind == "globals":
            self.globals = {k: synth.as_u16(v) for k, v in t.items()}
            H = self.shape.hidden
            for r in self.rows:
                self.x[r] = bits_to_f32(self.globals["embed"][int(self.tokens[r])]).copy()
        elif kind == "layer":
            self.layer_w = {k: synth.as_u16(v) for k, v in t.items()}
        elif kind == "kv":
            w1 = oracle.Weights(self.globals, [self.layer_w])

            def run(r):
                c = int(self.ctx[r])
                a = int(self.seq_start[r])
                nblk = (c + 1 + 15) // 16
                kv = oracle.PagedKV(self.cfg1, nblk, n_layers=1)
                table = np.arange(nblk, dtype=np.int32)[None, :]
                k = synth.as_u16(t["k"][a:a + c])
                v = synth.as_u16(t["v"][a:a + c])
                kv.fill(0, k, v, np.array([0, c], dtype=np.int32), table)
                tr = {} if layer in self.keep_layers else None
                att = oracle.layer_step(self.cfg1, w1.layer(0), self.x[r], c, kv.k[0], kv.v[0], table[0], want_attn=True, trace=tr)
                if tr is not None:
                    self.trace[layer][r] = tr
                return r, att
            if layer in self.keep_layers:
                self.x_before[layer] = {r: self.x[r].copy() for r in self.rows}
                self.trace[layer] = {}
                self.layer_bias[layer] = self.layer_w["bqkv"].copy()
            for r, att in self.pool.map(run, self.rows):
                self.attn[r].append(att)
            if os.environ.get("HX_PARITY_PROGRESS"):     # long every-row runs: one line per layer of oracle work
                print("oracle%s: layer %d of %d rows done" % (" (reordered)" if self.descending else "", layer, len(self.rows)), flush=True)
            if layer in self.keep_layers:
                self.x_after[layer] = {r: self.x[r].copy() for r in self.rows}
                # sum_k |x_k| |w_kn| of every product of the layer, per kept row: the scale of its fp32 rounding error
                tr = self.trace[layer]

                def mags(inp, *names):
                    xa = np.abs(np.stack([bits_to_f32(f32_to_bf16_bits_ref(tr[r][inp])) for r in self.rows]))
                    return [dict(zip(self.rows, xa @ np.abs(bits_to_f32(self.layer_w[n])))) for n in names]
                self.mag[layer] = dict(zip(("qkv", "o", "g", "u", "d"),
                                           mags("u1", "wqkv") + mags("o", "wo") + mags("u2", "wg", "wu") + mags("m", "wd")))

    def finish(self):
        if self.descending:
            with oracle.descending_sums():
                return self._finish()
        return self._finish()

    def _finish(self):
        cfg = oracle.make_config(self.shape)
        w = oracle.Weights(self.globals, [self.layer_w])      # only embed / gf / wlm are used by head()

        def run(r):
            return r, oracle.head(cfg, w, self.x[r])
        for r, (lg, tok) in self.pool.map(run, self.rows):
            self.logits[r], self.next[r] = lg, tok
        self.pool.shutdown()
        return self
