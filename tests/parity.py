"""Shared machinery of the GPU parity tests: the bars of the numeric contract, the comparison of one decode step
with the oracle, and the runner that builds a (possibly truncated) full-size workload on the GPU while the oracle
recomputes chosen rows layer by layer.

Bars (the numeric contract): max |logit error| <= 2e-2 * max|logit|; attention output max abs error <= 1e-2 in
every layer; greedy tokens agree.

Two evaluations of the oracle.  The contract rounds activations to bf16 at seven points per layer, so two correct
fp32 evaluations that differ only in summation order round a few activations differently and drift apart with depth.
The oracle built with every sum reversed (descending index order) is such a second evaluation; its distance from the
oracle on the same rows ("the floor") is measured on the CPU, independently of the GPU, and is used in three ways,
each of which involves only oracle quantities on the right-hand side:
  * a row on which the GPU picks another token than the oracle must be a near-tie BY THE ORACLE'S OWN LOGITS: the
    oracle's logit of the GPU's token lies within twice what the reordering moves that row's logits;
  * the GPU's error pooled over the rows (root mean square) must not exceed RMS_FACTOR times the reordered
    oracle's, so a systematic loss of precision shows even while every maximum is inside its bar;
  * at full depth only (28 / 48 layers), where the floor itself reaches the contract's bars, the bars become
    max(contract, FLOOR_FACTOR * floor).  Shallow runs (1 and 2 layers) are held to the contract bars alone.
"""
import dataclasses

import numpy as np
import torch

import oracle
from paper_2511_00796_amd import synth
from util import OracleRows

LOGIT_TOL = 2e-2
ATTN_TOL = 1e-2
FLOOR_FACTOR = 1.5
RMS_FACTOR = 1.5
TIE_REL = 1e-6        # without a floor: tokens may differ only where the oracle's two logits are an fp32 tie
# SiLU(gate) * up as bf16: one bf16 step of the oracle's value, plus this times (sum_k |x w_gate| + sum_k |x w_up|) for
# values near zero, where the fp32 reassociation error of gate and up (measured <= 3e-7 of those sums; silu' <= 1.1,
# |up| and |silu(gate)| of a few units) is no longer small against the value itself
GATE_UP_SLACK = 2e-6
ROPE_SLACK = 2e-6     # same reasoning for q and k after the rotation (a difference of two products of the projection)


@dataclasses.dataclass
class StepReport:
    logit_err: float            # max |gpu - oracle| / max|oracle logit|
    attn_err: float             # max abs attention-output error over all layers
    agreement: float            # fraction of rows with the oracle's greedy token
    floor_logit_err: float = 0.0
    floor_attn_err: float = 0.0
    floor_agreement: float = 1.0
    rms_ratio: float = 0.0      # rms(gpu - oracle) / rms(reordered - oracle), pooled over rows
    worst_row_rms_ratio: float = 0.0
    mismatches: list = dataclasses.field(default_factory=list)   # (row, oracle deficit of the GPU's token, bound)

    def line(self):
        s = "logit err / max|logit| %.3e, attention err %.3e, agreement %.4f" % (self.logit_err, self.attn_err, self.agreement)
        if self.floor_logit_err:
            s += (" | reordered oracle: %.3e, %.3e, %.4f | rms ratio %.2f (worst row %.2f)"
                  % (self.floor_logit_err, self.floor_attn_err, self.floor_agreement, self.rms_ratio, self.worst_row_rms_ratio))
        if self.mismatches:
            s += " | differing rows (row, deficit, bound): %s" % [(r, round(d, 5), round(b, 5)) for r, d, b in self.mismatches]
        return s


def compare_step(gpu_logits, gpu_tokens, gpu_attn, ref_logits, ref_tokens, ref_attn, what,
                 alt_logits=None, alt_tokens=None, alt_attn=None, floor_in_bars=False, rms_factor=RMS_FACTOR, quiet=False):
    """Apply the bars to one step.  alt_*: the reordered oracle on the same rows (None: no floor, tokens must agree
    unless the oracle's own logits tie to fp32 rounding).  floor_in_bars: full-depth runs."""
    scale = float(np.abs(ref_logits).max())
    lerr = float(np.abs(gpu_logits - ref_logits).max())
    aerr = float(np.abs(gpu_attn - ref_attn).max())
    rep = StepReport(lerr / scale, aerr, float((gpu_tokens == ref_tokens).mean()))
    bar_l, bar_a = LOGIT_TOL * scale, ATTN_TOL
    if alt_logits is not None:
        fl = float(np.abs(alt_logits - ref_logits).max())
        fa = float(np.abs(alt_attn - ref_attn).max())
        rep.floor_logit_err, rep.floor_attn_err = fl / scale, fa
        rep.floor_agreement = float((alt_tokens == ref_tokens).mean())
        if floor_in_bars:
            bar_l, bar_a = max(bar_l, FLOOR_FACTOR * fl), max(bar_a, FLOOR_FACTOR * fa)
        g2 = ((gpu_logits - ref_logits).astype(np.float64) ** 2).mean(axis=1)
        a2 = ((alt_logits - ref_logits).astype(np.float64) ** 2).mean(axis=1)
        rep.rms_ratio = float(np.sqrt(g2.mean() / max(a2.mean(), 1e-300)))
        rep.worst_row_rms_ratio = float(np.sqrt((g2 / np.maximum(a2, 1e-300)).max()))
    for b in np.nonzero(gpu_tokens != ref_tokens)[0]:
        deficit = float(ref_logits[b].max() - ref_logits[b][int(gpu_tokens[b])])
        bound = TIE_REL * scale if alt_logits is None else 2.0 * float(np.abs(alt_logits[b] - ref_logits[b]).max())
        rep.mismatches.append((int(b), deficit, bound))
    if not quiet:
        print("%s: %s" % (what, rep.line()))
    assert lerr <= bar_l, (what, "logits", lerr, bar_l, scale)
    assert aerr <= bar_a, (what, "attention", aerr, bar_a)
    for b, deficit, bound in rep.mismatches:
        assert deficit <= bound, (what, "row", b, "oracle deficit of the GPU's token", deficit, "bound", bound)
    if alt_logits is not None and rms_factor:
        assert rep.rms_ratio <= rms_factor, (what, "pooled rms of the logit error vs the reordered oracle's", rep.rms_ratio)
    return rep


def assert_tokens_agree_like_the_oracles_evaluations(rep, n_rows):
    """Every differing row has already been shown to be a near-tie by the oracle's own logits (compare_step).  This
    bounds how MANY there are: both counts are small-number statistics of the same population of near-tie rows, so the
    GPU may differ from the oracle on at most twice as many rows as the reordered oracle does, plus two."""
    gpu = round((1.0 - rep.agreement) * n_rows)
    alt = round((1.0 - rep.floor_agreement) * n_rows)
    assert gpu <= 2 * alt + 2, ("rows with another token: GPU %d, reordered oracle %d of %d" % (gpu, alt, n_rows))


def sample_rows(wl, n=16):
    """The shortest, the longest and seeded random further rows, `n` in all (rows are independent in the step)."""
    ctx = synth.context_lengths(wl)
    rows = {int(np.argmin(ctx)), int(np.argmax(ctx))}
    rng = np.random.default_rng(wl.seed)
    while len(rows) < min(wl.batch, n):
        rows.add(int(rng.integers(0, wl.batch)))
    return sorted(rows)


def run_sampled(hx, wl, n_layers, rows, with_floor=False, floor_in_bars=False, kv_fp8=False, keep_layers=(),
                rms_factor=RMS_FACTOR):
    """Build `wl` (truncated to n_layers if given) on the GPU, run ONE decode step, and compare `rows` with the oracle.
    with_floor: also run the reordered oracle on the same rows.  keep_layers: layers whose residual stream before and
    after is kept on the oracle side (for the layer-resynchronised checks).  Returns (StepReport, workload, OracleRows)."""
    from paper_2511_00796_amd import workload
    shape = wl.shape if n_layers is None else dataclasses.replace(wl.shape, n_layers=n_layers)
    ctx = synth.context_lengths(wl)
    seq_start = np.concatenate([[0], np.cumsum(ctx)]).astype(np.int64)
    tokens = synth.token_ids(wl, wl.batch)
    orc = OracleRows(shape, rows, ctx, seq_start, tokens, kv_fp8=kv_fp8, keep_layers=keep_layers)
    alt = OracleRows(shape, rows, ctx, seq_start, tokens, descending=True, kv_fp8=kv_fp8) if with_floor else None

    def tap(kind, layer, t):
        orc.tap(kind, layer, t)
        if alt:
            alt.tap(kind, layer, t)
    dw = workload.build(wl, n_layers=n_layers, tap=tap, kv_dtype=hx.HX_KV_FP8_E4M3 if kv_fp8 else hx.HX_KV_BF16)
    orc.finish()
    cap = torch.empty(shape.n_layers, wl.batch, shape.q_dim, dtype=torch.float32, device="cuda")
    dw.engine.set_attn_capture(cap)
    dw.step()
    torch.cuda.synchronize()
    dw.engine.set_attn_capture(None)
    gl = dw.logits[rows].cpu().numpy()
    gt = dw.next_tokens[rows].cpu().numpy()
    ga = cap[:, rows].cpu().numpy()
    del cap

    def gathered(o):
        return (np.stack([o.logits[r] for r in rows]), np.array([o.next[r] for r in rows], dtype=np.int32),
                np.stack([np.stack(o.attn[r]) for r in rows], axis=1))
    rl, rt, ra = gathered(orc)
    al = at = aa = None
    if alt:
        alt.finish()
        al, at, aa = gathered(alt)
    rep = compare_step(gl, gt, ga, rl, rt, ra, "%s, %d layers, %d rows" % (wl.name, shape.n_layers, len(rows)),
                       al, at, aa, floor_in_bars=floor_in_bars, rms_factor=rms_factor)
    # whole-batch properties that hold at any size
    assert torch.isfinite(dw.logits).all()
    assert torch.equal(dw.next_tokens.long(), torch.argmax(dw.logits, dim=1))
    return rep, dw, orc


def stagewise_layer(hx, dw, orc, layer, rows):
    """One layer at depth, stage by stage, through the single-stage hooks (the kernels and launch plans decode_step uses
    at this batch size).  Every stage is fed the ORACLE's input of that stage for `rows` (rows the oracle did not
    compute get copies: their caches are their own) and compared with the oracle's output of that stage, so nothing
    that earlier layers or earlier stages have rounded differently is carried along: stage-level bars apply at any
    depth.  The one exception is the append, which takes the GPU's own projection (the hook adds the bias itself).
    Bars: products |err| <= 1e-5 * sum_k |x_k w_kn|; bf16 results at most one bf16 step from the oracle's, on at most
    1 % of the elements; attention output <= 1e-3.  Returns a dict of the measured worst cases."""
    eng, s, B = dw.engine, dw.engine.shape, dw.wl.batch
    tr, mag = orc.trace[layer], orc.mag[layer]
    src = [b if b in tr else rows[b % len(rows)] for b in range(B)]

    def batch(name):
        pick = orc.x_before[layer] if name == "x_in" else None
        return torch.from_numpy(np.stack([pick[r] if pick is not None else tr[r][name] for r in src])).cuda()

    def got(t):
        return t[rows].cpu().numpy()

    def ref(name):
        return np.stack([tr[r][name] for r in rows])

    out = {}

    def product(name, y, want, scale):
        err = np.abs(y - want) / (np.stack([scale[r] for r in rows]) + 1e-30)
        out[name] = float(err.max())
        assert np.all(np.abs(y - want) <= 1e-5 * np.stack([scale[r] for r in rows]) + 1e-7), (layer, name, out[name])

    def rounded(name, y, want, slack=0.0):
        step = np.abs(want) * 2.0 ** -7 + slack + 1e-30
        assert np.all(np.abs(y - want) <= step), (layer, name, float((np.abs(y - want) / step).max()))
        out[name] = float(np.mean(y != want))
        assert out[name] <= 0.01, (layer, name, out[name])

    rounded("norm1", got(eng.stage_rmsnorm(hx.HX_T_G1, layer, batch("x_in"))), ref("u1"))
    y_qkv = eng.stage_linear(hx.HX_T_WQKV, layer, batch("u1"))
    bias = torch.from_numpy((orc.layer_bias[layer].astype(np.uint32) << 16).view(np.float32)).cuda()
    product("qkv", got(y_qkv + bias), ref("qkv"), mag["qkv"])
    q = eng.stage_rope_append(dw.kv, layer, y_qkv, dw.positions, dw.table_d)
    # the append starts from the GPU's projection, which differs from the oracle's by fp32 reassociation (measured
    # <= 3e-7 of sum_k |x w|); where a rotation cancels, that difference is no longer small against the result
    rot_slack = ROPE_SLACK * np.stack([mag["qkv"][r] for r in rows]).max(axis=1, keepdims=True)
    rounded("rope_q", got(q), ref("q"), slack=rot_slack)
    # what the append wrote: the block that holds the new position, read back through a one-block table
    pos = dw.ctx[rows].astype(np.int64)
    tb = np.ascontiguousarray(dw.table[rows, pos // 16][:, None]).astype(np.int32)
    start = (16 * np.arange(len(rows) + 1)).astype(np.int32)
    kg, vg = dw.kv.gather(layer, 16 * len(rows), torch.from_numpy(start).cuda(), torch.from_numpy(tb).cuda())
    sel = 16 * np.arange(len(rows)) + pos % 16
    rounded("append_k", kg.float().cpu().numpy()[sel].reshape(len(rows), -1), ref("k_new"), slack=rot_slack)
    rounded("append_v", vg.float().cpu().numpy()[sel].reshape(len(rows), -1), ref("v_new"), slack=rot_slack)
    att = got(eng.stage_attention(dw.kv, layer, batch("q"), dw.seq_lens_d, dw.table_d))
    out["attention"] = float(np.abs(att - ref("o")).max())
    assert out["attention"] <= 1e-3, (layer, out["attention"])
    product("o", got(eng.stage_linear(hx.HX_T_WO, layer, batch("o"))), ref("y_o"), mag["o"])
    rounded("norm2", got(eng.stage_rmsnorm(hx.HX_T_G2, layer, batch("x_mid"))), ref("u2"))
    g_slack = GATE_UP_SLACK * (np.stack([mag["g"][r] for r in rows]) + np.stack([mag["u"][r] for r in rows]))
    rounded("gate_up", got(eng.stage_linear(hx.HX_T_WG, layer, batch("u2"))), ref("m"), slack=g_slack)
    product("down", got(eng.stage_linear(hx.HX_T_WD, layer, batch("m"))), ref("y_d"), mag["d"])
    torch.cuda.synchronize()
    return out
