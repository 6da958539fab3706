"""What a rollout server does around the step, shown on the GPU through the C ABI: response groups sharing the
physical blocks of their prompt, sequences leaving and joining between steps, and a new policy version packed
into a live engine.  All of it rests on decode_step being a pure function of (weights, cache contents, inputs).
Each feature is checked twice: against the CPU oracle given the same block table / batch / weights (contract bars,
tokens equal), and for the bit-identity the feature promises between two ways of running the GPU path."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2511_00796_amd import synth
from parity import compare_step
from util import host_model

pytestmark = pytest.mark.gpu

SHAPE = dataclasses.replace(synth.TINY, name="serving", n_layers=2)


@pytest.fixture(scope="module")
def hx():
    from paper_2511_00796_amd import binding
    binding.load()
    assert torch.cuda.is_available()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def engine_with(hx, seed, max_batch=16, max_seq_len=512):
    eng = hx.Engine(SHAPE, max_batch, max_seq_len)
    for l in range(SHAPE.n_layers):
        eng.pack_layer(l, synth.layer_weights(SHAPE, l, seed))
    eng.pack_globals(synth.global_weights(SHAPE, seed))
    torch.cuda.synchronize()
    return eng


def step(eng, kv, tokens, ctx, table, want_attn=False):
    B = len(ctx)
    logits = torch.empty(B, SHAPE.vocab, dtype=torch.float32, device="cuda")
    nxt = torch.empty(B, dtype=torch.int32, device="cuda")
    ctx = np.asarray(ctx, dtype=np.int32)
    cap = torch.empty(SHAPE.n_layers, B, SHAPE.q_dim, dtype=torch.float32, device="cuda") if want_attn else None
    eng.set_attn_capture(cap)
    eng.decode_step(kv, dev(np.asarray(tokens, np.int32)), dev(ctx), dev(ctx + 1), dev(table), logits, nxt)
    torch.cuda.synchronize()
    eng.set_attn_capture(None)
    return (logits.cpu(), nxt.cpu(), cap.cpu()) if want_attn else (logits.cpu(), nxt.cpu())


def oracle_step(seed, data, start, table, n_blocks, tokens, ctx):
    """The oracle's step for the model of `seed` over a cache it fills itself from the same K/V rows through the same
    block table (any table: shared blocks are simply written once per sequence that names them)."""
    w, _, _ = host_model(SHAPE, seed)
    cfg = oracle.make_config(SHAPE)
    okv = oracle.PagedKV(cfg, n_blocks)
    for l, (k, v) in enumerate(data):
        okv.fill(l, synth.as_u16(k), synth.as_u16(v), start, table)
    ctx = np.asarray(ctx, dtype=np.int32)
    return oracle.decode_step(cfg, w, okv, np.asarray(tokens, np.int32), ctx, ctx + 1, table, want_attn=True)


def check_against_oracle(gpu, ref, what):
    (gl, gt, ga), (rl, rt, ra) = gpu, ref
    rep = compare_step(gl.numpy(), gt.numpy(), ga.numpy(), rl, rt, ra, what)
    assert rep.agreement == 1.0 or all(d <= b for _, d, b in rep.mismatches)


def test_response_groups_share_the_blocks_of_their_prompt(hx):
    """2 prompts x 3 responses.  Prompt length 48 = 3 full blocks.  Layout A gives every sequence private copies of
    its prompt's K/V; layout B maps the first three table entries of a group to the SAME physical blocks.  The step
    reads the same values either way, so logits and tokens are identical bit for bit, with 12 fewer blocks."""
    eng = engine_with(hx, 7)
    P, resp = 48, [5, 17, 30, 1, 16, 33]
    ctx = np.array([P + r for r in resp], dtype=np.int32)
    nblk = (ctx + 1 + 15) // 16
    rng = np.random.default_rng(11)
    kvd = SHAPE.n_kv_heads * SHAPE.head_dim
    total = int(ctx.sum())
    start = np.concatenate([[0], np.cumsum(ctx)]).astype(np.int32)
    tokens = rng.integers(0, SHAPE.vocab, size=6)

    def kv_data(layer):
        k = rng.normal(0, 1, size=(total, kvd)).astype(np.float32)
        v = rng.normal(0, 1, size=(total, kvd)).astype(np.float32)
        for grp in range(2):                               # the prompt part is common to the group's sequences
            first = 3 * grp
            for b in range(first + 1, first + 3):
                k[start[b]:start[b] + P] = k[start[first]:start[first] + P]
                v[start[b]:start[b] + P] = v[start[first]:start[first] + P]
        shp = (total, SHAPE.n_kv_heads, SHAPE.head_dim)
        return torch.from_numpy(k).to(torch.bfloat16).reshape(shp), torch.from_numpy(v).to(torch.bfloat16).reshape(shp)

    data = [kv_data(l) for l in range(SHAPE.n_layers)]
    width = int(nblk.max())
    # layout A: private blocks, shuffled
    nA = int(nblk.sum())
    permA = rng.permutation(nA)
    tableA = np.full((6, width), -1, dtype=np.int32)
    at = 0
    for b in range(6):
        tableA[b, :nblk[b]] = permA[at:at + nblk[b]]
        at += nblk[b]
    # layout B: blocks 0..2 of a group shared
    nB = nA - 2 * 2 * 3
    permB = list(rng.permutation(nB))
    tableB = np.full((6, width), -1, dtype=np.int32)
    for grp in range(2):
        shared = [permB.pop() for _ in range(3)]
        for b in range(3 * grp, 3 * grp + 3):
            tableB[b, :3] = shared
            tableB[b, 3:nblk[b]] = [permB.pop() for _ in range(nblk[b] - 3)]
    assert not permB
    outs = []
    for table, n in ((tableA, nA), (tableB, nB)):
        kv = hx.KVCache(eng, n)
        kv.pool.zero_()
        for l, (k, v) in enumerate(data):
            kv.prefill_fill(l, k.cuda(), v.cuda(), dev(start), dev(table))
        outs.append(step(eng, kv, tokens, ctx, table, want_attn=True))
        # the oracle over its own cache, filled through the same (private or shared-prefix) table
        check_against_oracle(outs[-1], oracle_step(7, data, start, table, n, tokens, ctx), "shared prefix, %d blocks" % n)
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert torch.isfinite(outs[0][0]).all()


def test_sequences_leave_and_join_between_steps(hx):
    """Step a batch of 6, then drop two sequences and admit a new one.  Every sequence's logits are those it gets
    when it is stepped alone: up to fp32 summation order, which the attention schedule (cut points depend on the
    whole batch) and the m-group of the products may change -- so tolerance, not equality; tokens must agree."""
    eng = engine_with(hx, 8)
    rng = np.random.default_rng(12)
    ctx_all = np.array([40, 300, 17, 129, 255, 64, 90], dtype=np.int32)
    nblk = (ctx_all + 1 + 15) // 16
    width = int(nblk.max())
    n = int(nblk.sum())
    perm = rng.permutation(n)
    table_all = np.full((7, width), -1, dtype=np.int32)
    at = 0
    for b in range(7):
        table_all[b, :nblk[b]] = perm[at:at + nblk[b]]
        at += nblk[b]
    start = np.concatenate([[0], np.cumsum(ctx_all)]).astype(np.int32)
    kv = hx.KVCache(eng, n)
    kv.pool.zero_()
    data = [synth.kv_fill(SHAPE, l, int(ctx_all.sum()), 99) for l in range(SHAPE.n_layers)]
    for l, (k, v) in enumerate(data):
        kv.prefill_fill(l, k.cuda(), v.cuda(), dev(start), dev(table_all))
    tokens_all = rng.integers(0, SHAPE.vocab, size=7)

    def run(rows, want_attn=False):
        rows = list(rows)
        return step(eng, kv, tokens_all[rows], ctx_all[rows], table_all[rows], want_attn)

    # the oracle steps all seven sequences once (rows are independent): every batch composition is compared with it
    rl, rt, ra = oracle_step(8, data, start, table_all, n, tokens_all, ctx_all)
    for rows in (list(range(6)), [0, 2, 3, 5, 6], [6]):
        check_against_oracle(run(rows, want_attn=True), (rl[rows], rt[rows], ra[:, rows]), "batch of rows %s" % rows)

    alone = [run([b]) for b in range(7)]        # each step re-writes the same K/V at position ctx: idempotent
    first = run(range(6))
    second = run([0, 2, 3, 5, 6])
    for rows, (logits, nxt) in ((list(range(6)), first), ([0, 2, 3, 5, 6], second)):
        for i, b in enumerate(rows):
            ref = alone[b][0][0]
            scale = float(ref.abs().max())
            assert float((logits[i] - ref).abs().max()) <= 1e-3 * scale, (b, float((logits[i] - ref).abs().max()), scale)
            assert int(nxt[i]) == int(alone[b][1][0])

    # What an RL consumer keeps of a step is the token drawn and its log-probability under the behaviour policy: the
    # same sequence sampled alone and inside a batch (same seed, same row id) draws the same token, and the
    # log-probabilities differ by no more than the logits do.
    def sample(rows):
        rows = list(rows)
        B = len(rows)
        ctx = ctx_all[rows]
        tok = torch.empty(B, dtype=torch.int32, device="cuda")
        lp = torch.empty(B, dtype=torch.float32, device="cuda")
        eng.decode_step_sample(kv, dev(tokens_all[rows].astype(np.int32)), dev(ctx), dev(ctx + 1), dev(table_all[rows]), 0.8, 2024,
                               None, tok, lp, row_ids=dev(np.array(rows, dtype=np.int32)))
        torch.cuda.synchronize()
        return tok.cpu().numpy(), lp.cpu().numpy()

    together_tok, together_lp = sample(range(6))
    for i, b in enumerate(range(6)):
        tok, lp = sample([b])
        assert int(tok[0]) == int(together_tok[i]), b
        assert abs(float(lp[0]) - float(together_lp[i])) <= 2e-3, (b, float(lp[0]), float(together_lp[i]))


def test_new_policy_version_packed_into_a_live_engine(hx):
    """hx_weights_pack overwrites the streaming-layout weights in place: after packing version B the engine is
    indistinguishable (bit for bit) from one created with B, and packing A again restores A's outputs."""
    rng = np.random.default_rng(13)
    ctx = np.array([33, 100, 7], dtype=np.int32)
    nblk = (ctx + 1 + 15) // 16
    table, n = synth.block_table(ctx + 1, 16, 3)
    start = np.concatenate([[0], np.cumsum(ctx)]).astype(np.int32)
    tokens = rng.integers(0, SHAPE.vocab, size=3)

    data = [synth.kv_fill(SHAPE, l, int(ctx.sum()), 5) for l in range(SHAPE.n_layers)]

    def cache_for(eng):
        kv = hx.KVCache(eng, n)
        kv.pool.zero_()
        for l, (k, v) in enumerate(data):
            kv.prefill_fill(l, k.cuda(), v.cuda(), dev(start), dev(table))
        return kv

    def pack(eng, seed):
        for l in range(SHAPE.n_layers):
            eng.pack_layer(l, synth.layer_weights(SHAPE, l, seed))
        eng.pack_globals(synth.global_weights(SHAPE, seed))
        torch.cuda.synchronize()

    live = engine_with(hx, 21)
    out_a = step(live, cache_for(live), tokens, ctx, table)
    fresh_b = engine_with(hx, 22)
    out_b = step(fresh_b, cache_for(fresh_b), tokens, ctx, table)
    assert not torch.equal(out_a[0], out_b[0])
    pack(live, 22)
    swapped = step(live, cache_for(live), tokens, ctx, table, want_attn=True)
    assert torch.equal(swapped[0], out_b[0]) and torch.equal(swapped[1], out_b[1])
    # ... and it computes what the oracle computes with version B's weights (and no longer what it computes with A's)
    ref_b = oracle_step(22, data, start, table, n, tokens, ctx)
    check_against_oracle(swapped, ref_b, "live engine after packing version B")
    ref_a = oracle_step(21, data, start, table, n, tokens, ctx)
    assert float(np.abs(swapped[0].numpy() - ref_a[0]).max()) > 0.1 * float(np.abs(ref_a[0]).max())
    pack(live, 21)
    back = step(live, cache_for(live), tokens, ctx, table, want_attn=True)
    assert torch.equal(back[0], out_a[0])
    check_against_oracle(back, ref_a, "live engine after packing version A again")


def test_device_side_inputs_are_validated_without_running_the_step(hx):
    """decode_step trusts its device arrays; hx_validate_step_inputs turns a bad token, position, length or block id
    into an error that names the first offending row.  Only the validator runs on the bad inputs."""
    eng = engine_with(hx, 9, max_batch=8, max_seq_len=200)
    ctx = np.array([10, 150, 33, 64], dtype=np.int32)
    table, n = synth.block_table(ctx + 1, 16, 4)
    kv = hx.KVCache(eng, n)
    tokens = np.array([1, 2, 3, 4], dtype=np.int32)

    def check(tok=tokens, pos=ctx, lens=ctx + 1, tab=table):
        eng.validate_step_inputs(kv, dev(np.asarray(tok, np.int32)), dev(np.asarray(pos, np.int32)),
                                 dev(np.asarray(lens, np.int32)), dev(np.asarray(tab, np.int32)))

    check()                                                   # the good inputs pass
    bad = tokens.copy(); bad[2] = SHAPE.vocab
    with pytest.raises(hx.HexError, match="row 2: token id"):
        check(tok=bad)
    bad = tokens.copy(); bad[1] = -1; bad[3] = -5
    with pytest.raises(hx.HexError, match="row 1: token id -1"):
        check(tok=bad)
    pos = ctx.copy(); pos[0] = 200                            # == max_seq_len
    with pytest.raises(hx.HexError, match="row 0: position 200"):
        check(pos=pos, lens=pos + 1)
    pos = ctx.copy(); pos[1] = table.shape[1] * 16            # beyond the table's columns
    with pytest.raises(hx.HexError, match="row 1: position"):
        check(pos=pos, lens=pos + 1)
    lens = ctx + 1; lens[3] += 1
    with pytest.raises(hx.HexError, match="row 3: seq_len 66 is not position"):
        check(lens=lens)
    tab = table.copy(); tab[1, 4] = n                         # one past the pool
    with pytest.raises(hx.HexError, match="row 1: a block id"):
        check(tab=tab)
    tab = table.copy(); tab[2, 0] = -1
    with pytest.raises(hx.HexError, match="row 2: a block id"):
        check(tab=tab)
    tab = table.copy(); tab[0, 3] = -7                        # past ceil(seq_len / 16) entries of row 0: ignored
    check(tab=tab)


def test_two_engines_over_one_copy_of_the_weights_on_two_streams(hx):
    """A second engine wraps the first one's packed weights with a workspace of its own; the two process different
    prompts concurrently on two streams.  Each must leave exactly the cache, and produce exactly the logits, that
    a single engine produces for the same calls alone: the step keeps no state outside its workspace and cache."""
    a = engine_with(hx, 21, max_batch=64, max_seq_len=400)
    b = hx.Engine(SHAPE, 64, 400, weights=a.weights)
    rng = np.random.default_rng(5)
    n_tok = [300, 260]
    prompts = [rng.integers(0, SHAPE.vocab, size=n).astype(np.int32) for n in n_tok]
    tables, pools = [], []
    for n in n_tok:
        t, nb = synth.block_table(np.array([n + 1]), 16, 40 + n)
        tables.append((t, nb))

    def process(eng, i, stream):
        t, nb = tables[i]
        kv = hx.KVCache(eng, nb)
        with torch.cuda.stream(stream):
            kv.pool.zero_()
            for at in range(0, n_tok[i] - 1, 64):
                ps = np.arange(at, min(at + 64, n_tok[i] - 1), dtype=np.int32)
                eng.prefill_chunk(kv, dev(prompts[i][ps]), dev(ps), dev(ps + 1), dev(np.repeat(t, len(ps), axis=0)))
            logits = torch.empty(1, SHAPE.vocab, dtype=torch.float32, device="cuda")
            nxt = torch.empty(1, dtype=torch.int32, device="cuda")
            pos = np.array([n_tok[i] - 1], dtype=np.int32)
            eng.decode_step(kv, dev(prompts[i][-1:]), dev(pos), dev(pos + 1), dev(t), logits, nxt)
        return kv, logits, nxt

    main = torch.cuda.current_stream()
    alone = []
    for i in range(2):                                   # one engine, one stream, one prompt after the other
        kv, logits, nxt = process(a, i, main)
        torch.cuda.synchronize()
        alone.append((kv.pool.clone(), logits.clone(), nxt.clone()))
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    together = [process(a, 0, s1), process(b, 1, s2)]    # both in flight at once
    torch.cuda.synchronize()
    for i in range(2):
        kv, logits, nxt = together[i]
        assert torch.equal(kv.pool, alone[i][0]), i
        assert torch.equal(logits, alone[i][1]) and torch.equal(nxt, alone[i][2]), i
    assert torch.isfinite(together[0][1]).all() and torch.isfinite(together[1][1]).all()
