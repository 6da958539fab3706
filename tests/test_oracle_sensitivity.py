"""How far two CORRECT fp32 evaluations of the decode step drift apart, on the CPU.

The oracle adds the terms of every sum (matrix products, mean of squares, score dot products, softmax
denominator, probability-weighted sum of V) in ascending index order; built with -DORC_SUM_DESCENDING it
adds them in descending order.  Both are valid "bf16 in, fp32 accumulate" evaluations of the same step.
Within a layer they agree to fp32 rounding; but a few activations land on opposite sides of a bf16
rounding boundary (the first ones at the attention output of the first layer), each such flip perturbs
everything downstream, and the random-weight network amplifies the perturbation from layer to layer.  This pins the mechanism behind the depth-dependent tolerance of
the full-size GPU parity tests: it is a property of the numeric contract, not of an implementation."""
import dataclasses

import numpy as np

import oracle
from paper_2511_00796_amd import synth
from util import host_model


def drift(n_layers):
    shape = synth.ModelShape("drift", n_layers, 256, 4, 2, 64, 688, 1024)
    w, _, _ = host_model(shape, 31)
    cfg = oracle.make_config(shape)
    ctx = np.array([40, 77, 150, 231], dtype=np.int32)
    table, nb = synth.block_table(ctx + 1, 16, 3)
    start = np.concatenate([[0], np.cumsum(ctx)]).astype(np.int32)
    toks = np.array([5, 77, 901, 333], dtype=np.int32)
    out = []
    for desc in (False, True):
        kv = oracle.PagedKV(cfg, nb)
        for l in range(n_layers):
            k, v = synth.kv_fill(shape, l, int(ctx.sum()), 9)
            kv.fill(l, synth.as_u16(k), synth.as_u16(v), start, table)
        if desc:
            with oracle.descending_sums():
                out.append(oracle.decode_step(cfg, w, kv, toks, ctx, ctx + 1, table)[0])
        else:
            out.append(oracle.decode_step(cfg, w, kv, toks, ctx, ctx + 1, table)[0])
    return float(np.abs(out[0] - out[1]).max() / np.abs(out[0]).max())


def test_reordered_sums_agree_after_one_layer_and_drift_with_depth():
    d1, d28 = drift(1), drift(28)
    print("relative logit drift between ascending and descending sums: 1 layer %.2e, 28 layers %.2e" % (d1, d28))
    assert d1 <= 5e-3                 # a handful of bf16 flips at most
    assert d28 >= 1.5 * d1            # amplified by depth (this small model saturates near 4e-3)
    assert d28 <= 1e-1                # ... but still the same function
