"""Pins of the oracle's whole decode step: a library implementation of the same decoder family
(transformers' Qwen2 on CPU, fp32), brute-force dense causal recomputation, paging and batch
invariances, and closed-form special cases.  CPU only."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from oracle import make_config
from paper_2511_00796_amd import synth
from util import bits_to_f32, host_model

SMALL = synth.ModelShape("pin", 2, 128, 4, 2, 32, 176, 320)


def prefill_by_decode(cfg, w, tokens_per_seq, table, num_blocks, want_attn=False):
    """Feed each sequence's tokens one position at a time through decode_step (all sequences in
    lock step while they last).  Returns per-sequence list of logits rows (+ attn rows)."""
    B = len(tokens_per_seq)
    kv = oracle.PagedKV(cfg, num_blocks)
    out = [[] for _ in range(B)]
    att = [[] for _ in range(B)]
    for pos in range(max(len(t) for t in tokens_per_seq)):
        live = [b for b in range(B) if pos < len(tokens_per_seq[b])]
        toks = np.array([tokens_per_seq[b][pos] for b in live], dtype=np.int32)
        p = np.full(len(live), pos, dtype=np.int32)
        logits, nxt, attn = oracle.decode_step(cfg, w, kv, toks, p, p + 1, table[live], want_attn=want_attn)
        for i, b in enumerate(live):
            out[b].append(logits[i])
            if want_attn:
                att[b].append(attn[:, i])
    return out, att, kv


def test_full_causal_matches_transformers_qwen2_fp32():
    """The dense recomputation with the bf16 rounding points switched off is the same function
    as the library's Qwen2 decoder in fp32 (eager attention): pins RoPE pairing and base, GQA
    head mapping, bias placement, norm placement, SwiGLU and the LM head orientation."""
    from transformers import Qwen2Config, Qwen2ForCausalLM
    s = SMALL
    w, g, layers = host_model(s, 11)
    hf_cfg = Qwen2Config(vocab_size=s.vocab, hidden_size=s.hidden, intermediate_size=s.intermediate,
                         num_hidden_layers=s.n_layers, num_attention_heads=s.n_q_heads,
                         num_key_value_heads=s.n_kv_heads, max_position_embeddings=4096,
                         rms_norm_eps=s.rms_eps, rope_theta=s.rope_theta, tie_word_embeddings=False,
                         attn_implementation="eager", use_sliding_window=False)
    model = Qwen2ForCausalLM(hf_cfg).float().eval()
    f = lambda bits: torch.from_numpy(bits_to_f32(bits).copy())
    sd = {"model.embed_tokens.weight": f(g["embed"]), "model.norm.weight": f(g["gf"]),
          "lm_head.weight": f(g["wlm"]).t().contiguous()}
    qd, kd = s.q_dim, s.kv_dim
    for l, lw in enumerate(layers):
        p = f"model.layers.{l}."
        wqkv, bqkv = f(lw["wqkv"]), f(lw["bqkv"])
        sd[p + "self_attn.q_proj.weight"] = wqkv[:, :qd].t().contiguous()
        sd[p + "self_attn.k_proj.weight"] = wqkv[:, qd:qd + kd].t().contiguous()
        sd[p + "self_attn.v_proj.weight"] = wqkv[:, qd + kd:].t().contiguous()
        sd[p + "self_attn.q_proj.bias"] = bqkv[:qd].clone()
        sd[p + "self_attn.k_proj.bias"] = bqkv[qd:qd + kd].clone()
        sd[p + "self_attn.v_proj.bias"] = bqkv[qd + kd:].clone()
        sd[p + "self_attn.o_proj.weight"] = f(lw["wo"]).t().contiguous()
        sd[p + "mlp.gate_proj.weight"] = f(lw["wg"]).t().contiguous()
        sd[p + "mlp.up_proj.weight"] = f(lw["wu"]).t().contiguous()
        sd[p + "mlp.down_proj.weight"] = f(lw["wd"]).t().contiguous()
        sd[p + "input_layernorm.weight"] = f(lw["g1"])
        sd[p + "post_attention_layernorm.weight"] = f(lw["g2"])
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in m or "inv_freq" in m for m in missing), (missing, unexpected)
    # positions far from zero matter for RoPE: use a long-ish sequence
    toks = np.random.default_rng(3).integers(0, s.vocab, size=300).astype(np.int32)
    with torch.no_grad():
        ref = model(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    got, _ = oracle.full_causal(make_config(s, round_act=False), w, toks)
    assert np.abs(got - ref).max() <= 2e-4 * max(1.0, np.abs(ref).max())
    # the rounding points move the logits by bf16-sized amounts only
    got_r, _ = oracle.full_causal(make_config(s, round_act=True), w, toks)
    assert 0 < np.abs(got_r - ref).max() <= 3e-2 * np.abs(ref).max()


def test_stepwise_decode_equals_dense_causal_recomputation_bit_for_bit():
    """Config-1 protocol on the tiny shape: prompts of 32..128 tokens then 16 more positions, fed
    token by token through the paged cache with a shuffled table, against recomputing the whole
    sequence densely without any cache."""
    wl = synth.WORKLOADS["tiny-b4"]
    s = wl.shape
    w, _, _ = host_model(s, wl.seed)
    cfg = make_config(s)
    ctx = synth.context_lengths(wl)
    n = ctx + wl.decode_steps
    assert n.max() <= 144
    toks = [synth.token_ids(wl, int(n[b]), salt=b) for b in range(wl.batch)]
    table, num_blocks = synth.block_table(n, s.block_size, wl.seed)
    step_logits, step_attn, _ = prefill_by_decode(cfg, w, toks, table, num_blocks, want_attn=True)
    for b in range(wl.batch):
        dense, dense_attn = oracle.full_causal(cfg, w, toks[b], want_attn=True)
        assert np.array_equal(np.stack(step_logits[b]), dense)
        assert np.array_equal(np.stack(step_attn[b], axis=1), dense_attn)


def test_step_invariant_to_block_permutation_block_size_and_batch_mates():
    s = SMALL
    w, _, _ = host_model(s, 5)
    rng = np.random.default_rng(9)
    lens = np.array([40, 9, 23], dtype=np.int32)
    toks = [rng.integers(0, s.vocab, size=int(n)).astype(np.int32) for n in lens]
    ref = None
    for bs, shuffle, seed in ((16, False, 0), (16, True, 1), (16, True, 2), (1, True, 3), (64, False, 0)):
        cfg = make_config(s, block_size=bs)
        table, nb = synth.block_table(lens, bs, seed, shuffle=shuffle)
        out, _, _ = prefill_by_decode(cfg, w, toks, table, nb)
        last = np.stack([o[-1] for o in out])
        if ref is None:
            ref = last
        assert np.array_equal(ref, last)
    # a row's result does not depend on which other rows share the batch
    cfg = make_config(s)
    table, nb = synth.block_table(lens[:1], 16, 0)
    solo, _, _ = prefill_by_decode(cfg, w, toks[:1], table, nb)
    assert np.array_equal(solo[0][-1], ref[0])


def test_zero_output_projections_reduce_the_step_to_norm_and_lm_head():
    s = SMALL
    w, g, layers = host_model(s, 21)
    for lw in layers:
        lw["wo"][:] = 0
        lw["wd"][:] = 0
    w = oracle.Weights(g, layers)
    cfg = make_config(s)
    table, nb = synth.block_table(np.array([1], dtype=np.int32), 16, 0)
    kv = oracle.PagedKV(cfg, nb)
    tok = 77
    logits, nxt, _ = oracle.decode_step(cfg, w, kv, [tok], [0], [1], table)
    e = bits_to_f32(g["embed"][tok]).astype(np.float64)
    u = e / np.sqrt((e ** 2).mean() + s.rms_eps) * bits_to_f32(g["gf"])
    u = torch.from_numpy(u.astype(np.float32)).to(torch.bfloat16).double().numpy()
    ref = u @ bits_to_f32(g["wlm"]).astype(np.float64)
    # u may differ from the oracle's by one bf16 ulp on a few elements (fp32 vs fp64 norm)
    assert np.abs(logits[0] - ref).max() <= 2e-3 * np.abs(ref).max()
    assert nxt[0] == int(np.argmax(logits[0]))


def test_planted_lm_head_column_wins_the_greedy_token():
    s = SMALL
    w, g, layers = host_model(s, 22)
    cfg = make_config(s)
    table, nb = synth.block_table(np.array([3], dtype=np.int32), 16, 0)
    toks = [np.array([5, 6, 7], dtype=np.int32)]
    base, _, _ = prefill_by_decode(cfg, w, toks, table, nb)
    col = 211
    # make column `col` of the LM head a large multiple of the final normalised activation's sign
    x_probe = base[0][-1]
    assert int(np.argmax(x_probe)) != col
    wl = bits_to_f32(g["wlm"]).copy()
    best = int(np.argmax(x_probe))
    wl[:, col] = wl[:, best] * 4.0          # 4x the winning column: exact in bf16, logit becomes 4x
    g2 = dict(g)
    g2["wlm"] = synth.as_u16(torch.from_numpy(wl).to(torch.bfloat16))
    w2 = oracle.Weights(g2, layers)
    out, _, _ = prefill_by_decode(cfg, w2, toks, table, nb)
    assert x_probe[best] > 0
    assert int(np.argmax(out[0][-1])) == col
    assert out[0][-1][col] == pytest.approx(4.0 * x_probe[best], rel=1e-6)


def test_decode_step_rejects_inconsistent_lengths():
    s = SMALL
    w, _, _ = host_model(s, 1)
    cfg = make_config(s)
    table, nb = synth.block_table(np.array([4], dtype=np.int32), 16, 0)
    kv = oracle.PagedKV(cfg, nb)
    with pytest.raises(ValueError):
        oracle.decode_step(cfg, w, kv, [1], [2], [2], table)


def test_new_token_is_cached_at_its_position_and_attended():
    """After a step at position p the pool holds the rounded k/v of that token at (table[p/bs], p%bs),
    and the next step's attention sees it: compare a two-step decode with the dense recomputation
    (covered above) and check the written slot directly."""
    s = SMALL
    w, _, _ = host_model(s, 2)
    cfg = make_config(s)
    lens = np.array([18], dtype=np.int32)
    table, nb = synth.block_table(lens, 16, 4)
    toks = [np.random.default_rng(1).integers(0, s.vocab, size=18).astype(np.int32)]
    _, _, kv = prefill_by_decode(cfg, w, toks, table, nb)
    used = set(table[0, :2].tolist())
    for blk in range(nb):
        filled = kv.k[0][blk].any(axis=(1, 2))
        if blk == table[0, 0]:
            assert filled.all()
        elif blk == table[0, 1]:
            assert filled[:2].all() and not filled[2:].any()
        else:
            assert not filled.any()
