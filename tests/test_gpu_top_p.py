"""GPU parity of decode_step_top_p against the oracle's nucleus sampler.

As for the temperature sampler the comparison is made on IDENTICAL logits (those the GPU step returns).  Two
integers are decided by floating point: the size of the kept set (the GPU accumulates mass in 2^-40 fixed point from
fp32 exp, the oracle in double) and the drawn token (fp32 perturbed scores on both sides).  The size must be equal
wherever the oracle's deciding running mass is further than 1e-7 from top_p; nearer than that one boundary entry
(plus its exact ties) may go either way.  The token must be equal unless the oracle's best and runner-up perturbed
scores are closer than 1e-4, or the sizes legitimately differ."""
import dataclasses

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

import oracle
from paper_2511_00796_amd import synth
from util import bits_to_f32

pytestmark = pytest.mark.gpu

LOGPROB_TOL = 2e-4          # fp32 z and max, fixed-point mass, against the oracle's fp64
GAP_TOL = 1e-4
MARGIN_TOL = 1e-7           # relative accuracy of a sum of ~1e5 fp32 exp() values


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.fixture(scope="module")
def hx():
    from paper_2511_00796_amd import binding
    binding.load()
    assert torch.cuda.is_available()
    return binding


def top_p_once(dw, temperature, top_p, seed, row_ids=None, want_sizes=True):
    B = dw.tokens.numel()
    tok = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    lp = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
    n = torch.full((B,), -1, dtype=torch.int32, device="cuda") if want_sizes else None
    dw.engine.decode_step_top_p(dw.kv, dw.tokens, dw.positions, dw.seq_lens_d, dw.table_d, temperature, top_p, seed,
                                dw.logits, tok, lp, row_ids, n)
    torch.cuda.synchronize()
    return tok.cpu().numpy(), lp.cpu().numpy(), (n.cpu().numpy() if want_sizes else None), dw.logits.cpu().numpy()


def check_against_oracle(tok, lp, n, logits, temperature, top_p, seed, rows, positions, what):
    otok, olp, on, margin, gap = oracle.sample_top_p(logits, temperature, top_p, seed, rows, positions)
    firm = margin > MARGIN_TOL
    assert np.array_equal(n[firm], on[firm]), (what, n[firm], on[firm])
    # where the cut is undecided in fp the sizes differ by the boundary entry and its exact ties only
    z = logits * (np.float32(1.0) / np.float32(temperature))
    for b in np.nonzero(n != on)[0]:
        srt = np.sort(z[b])[::-1]
        lo, hi = sorted((int(n[b]), int(on[b])))
        assert np.all(srt[lo:hi] == srt[lo]) and (lo == 0 or srt[lo - 1] > srt[lo]), (what, "row", int(b), lo, hi)
    same_set = n == on
    for b in np.nonzero((tok != otok) & same_set)[0]:
        assert gap[b] < GAP_TOL, (what, "row", int(b), "gap", float(gap[b]), int(tok[b]), int(otok[b]))
    same = (tok == otok) & same_set
    assert same.mean() >= 0.995, (what, float(same.mean()))
    err = float(np.abs(lp[same] - olp[same]).max())
    assert err <= LOGPROB_TOL, (what, err)
    # every drawn token lies in the GPU's own kept set: its z is among the n largest of its row
    for b in range(len(tok)):
        assert z[b, tok[b]] >= np.partition(z[b], -int(n[b]))[-int(n[b])], (what, "row", int(b))
    return float(same.mean()), err, float(same_set.mean())


@pytest.mark.parametrize("temperature,top_p", [(1.0, 0.9), (0.6, 0.5), (1.7, 0.95), (0.8, 0.02)])
def test_nucleus_step_matches_oracle_on_the_same_logits(hx, temperature, top_p):
    """1.5B-shaped layers (2 of them; vocab 151 936, not a multiple of the 2 048 histogram bins or of 1 024
    threads), batch 48: kept-set sizes, tokens and log-probabilities; the logits equal those of the greedy step."""
    from paper_2511_00796_amd import workload
    wl = dataclasses.replace(synth.WORKLOADS["1.5b-b64"], batch=48, lo=64, hi=1500)
    dw = workload.build(wl, n_layers=2)
    dw.step()
    torch.cuda.synchronize()
    greedy_logits = dw.logits.clone()
    seed = 2 ** 35 + 777
    tok, lp, n, logits = top_p_once(dw, temperature, top_p, seed)
    assert torch.equal(greedy_logits.cpu(), torch.from_numpy(logits))
    pos = dw.positions.cpu().numpy()
    agree, lperr, firm = check_against_oracle(tok, lp, n, logits, temperature, top_p, seed, np.arange(48), pos,
                                              "T=%g p=%g" % (temperature, top_p))
    print("top-p T=%g p=%g: agreement %.4f, max |logprob err| %.2e, kept %d..%d of %d, equal sizes %.2f"
          % (temperature, top_p, agree, lperr, n.min(), n.max(), logits.shape[1], firm))
    assert 1 <= n.min() and n.max() < logits.shape[1]
    # deterministic; other row ids give the oracle's draw for those ids; sizes are optional
    tok2, lp2, n2, _ = top_p_once(dw, temperature, top_p, seed)
    assert np.array_equal(tok, tok2) and np.array_equal(lp, lp2) and np.array_equal(n, n2)
    ids = torch.arange(500, 548, dtype=torch.int32, device="cuda")
    tok3, lp3, n3, _ = top_p_once(dw, temperature, top_p, seed, ids)
    assert np.array_equal(n3, n)                      # the kept set does not depend on the noise
    check_against_oracle(tok3, lp3, n3, logits, temperature, top_p, seed, np.arange(500, 548), pos, "row ids")
    tok4, lp4, _, _ = top_p_once(dw, temperature, top_p, seed, want_sizes=False)
    assert np.array_equal(tok4, tok) and np.array_equal(lp4, lp)


def test_top_p_one_is_the_temperature_sampler(hx):
    from paper_2511_00796_amd import workload
    wl = dataclasses.replace(synth.WORKLOADS["1.5b-b64"], batch=32, lo=64, hi=600)
    dw = workload.build(wl, n_layers=1)
    tok, lp, _, _ = top_p_once(dw, 0.9, 1.0, 4321, want_sizes=False)
    t0 = torch.zeros(32, dtype=torch.int32, device="cuda")
    l0 = torch.zeros(32, dtype=torch.float32, device="cuda")
    dw.engine.decode_step_sample(dw.kv, dw.tokens, dw.positions, dw.seq_lens_d, dw.table_d, 0.9, 4321, None, t0, l0)
    torch.cuda.synchronize()
    assert np.array_equal(tok, t0.cpu().numpy()) and np.array_equal(lp, l0.cpu().numpy())


def test_full_size_nucleus_step_7b_batch_128(hx):
    """The configuration the benchmark times (Qwen2-7B shape, batch 128, vocab 152 064): every row against the
    oracle's nucleus sampler on the step's own logits."""
    from paper_2511_00796_amd import workload
    dw = workload.build(synth.WORKLOADS["7b-b128"])
    seed = 2511007965
    tok, lp, n, logits = top_p_once(dw, 0.8, 0.9, seed)
    pos = dw.positions.cpu().numpy()
    agree, lperr, firm = check_against_oracle(tok, lp, n, logits, 0.8, 0.9, seed, np.arange(128), pos, "7b-b128")
    print("7b-b128 top-p 0.9: agreement %.4f, max |logprob err| %.2e, kept %d..%d, mean logprob %.3f"
          % (agree, lperr, n.min(), n.max(), float(lp.mean())))
    del dw
    torch.cuda.empty_cache()


def test_ties_at_the_cut_are_all_kept(hx):
    """LM head with five identical columns that dominate the row: the first of them alone exceeds top_p = 0.1, and
    all five are kept (their logits are bit-equal); each is drawn about equally often over 4 000 positions and
    the log-probability is log(1/5)."""
    shape = synth.ModelShape("stage-d128-g7", 1, 512, 14, 2, 128, 1376, 2048)
    eng = hx.Engine(shape, 64, 64)
    gw = synth.global_weights(shape, 4)
    wlm = gw["wlm"].clone()
    cols = [37, 38, 900, 1500, 2047]
    for c in cols[1:]:
        wlm[:, c] = wlm[:, cols[0]]
    for c in cols:
        wlm[:, c] *= 16
    gw["wlm"] = wlm
    eng.pack_globals(gw)
    x = np.abs(np.random.default_rng(3).normal(0, 1, size=(1, shape.hidden))).astype(np.float32)
    x = x * np.sign(bits_to_f32(synth.as_u16(wlm[:, cols[0]])))[None, :]
    x = np.repeat(x, 64, axis=0)
    counts = np.zeros(len(cols), dtype=np.int64)
    total = 0
    for rep in range(63):
        pos = torch.arange(rep * 64, rep * 64 + 64, dtype=torch.int32, device="cuda")
        y, tok, lp, n = eng.stage_lm_head_top_p(dev(x), pos, 1.0, 0.1, 99)
        y, tok, lp, n = y.cpu().numpy(), tok.cpu().numpy(), lp.cpu().numpy(), n.cpu().numpy()
        if rep == 0:
            assert all(np.all(y[:, c] == y[:, cols[0]]) for c in cols)
            p = scipy.special.softmax(y[0].astype(np.float64))
            assert p[cols[0]] > 0.1 and y[0].argmax() in cols
            otok, olp, on, _, _ = oracle.sample_top_p(y, 1.0, 0.1, 99, np.arange(64), pos.cpu().numpy())
            assert np.array_equal(otok, tok) and np.all(on == len(cols))
        assert np.all(n == len(cols)), n
        assert np.all(np.isin(tok, cols))
        assert np.allclose(lp, np.log(1.0 / len(cols)), atol=1e-5)
        counts += np.array([(tok == c).sum() for c in cols])
        total += 64
    expect = total / len(cols)
    assert float(((counts - expect) ** 2 / expect).sum()) < scipy.stats.chi2.ppf(0.9999, len(cols) - 1), counts


def test_tiny_config_draws_follow_the_renormalised_kept_set(hx):
    """Config-1 model (vocab 1024, batch 4), one fixed state, 5 000 seeds: no draw outside the kept set, and the
    kept entries appear with p_i / mass (chi-square over the 10 most likely + the rest of the set)."""
    from paper_2511_00796_amd import workload
    wl = dataclasses.replace(synth.WORKLOADS["tiny-b4"], kv_fill="normal")
    dw = workload.build(wl)
    T, top_p, n_seeds = 0.2, 0.5, 5000
    toks = np.zeros((n_seeds, 4), dtype=np.int64)
    tok = torch.zeros(4, dtype=torch.int32, device="cuda")
    lp = torch.zeros(4, dtype=torch.float32, device="cuda")
    n = torch.zeros(4, dtype=torch.int32, device="cuda")
    for s in range(n_seeds):
        dw.engine.decode_step_top_p(dw.kv, dw.tokens, dw.positions, dw.seq_lens_d, dw.table_d, T, top_p, 5000 + s,
                                    dw.logits, tok, lp, None, n)
        toks[s] = tok.cpu().numpy()
    logits = dw.logits.cpu().numpy()
    sizes = n.cpu().numpy()
    for b in range(4):
        p = scipy.special.softmax(logits[b].astype(np.float64) * float(np.float32(1.0) / np.float32(T)))
        order = np.argsort(-p, kind="stable")
        size = int(np.searchsorted(np.cumsum(p[order]), top_p) + 1)
        assert sizes[b] == size and 1 < size < 1024, (b, sizes[b], size)
        kept = order[:size]
        assert np.all(np.isin(toks[:, b], kept))
        q = p[kept] / p[kept].sum()
        k = min(10, size - 1)
        top = kept[:k]
        counts = np.array([(toks[:, b] == t).sum() for t in top] + [np.isin(toks[:, b], top, invert=True).sum()], dtype=np.float64)
        expect = np.array(list(q[:k]) + [1.0 - q[:k].sum()]) * n_seeds
        chi2 = float(((counts - expect) ** 2 / expect).sum())
        assert chi2 < scipy.stats.chi2.ppf(0.9999, len(expect) - 1), (b, chi2)


def test_top_p_arguments_are_validated(hx):
    from paper_2511_00796_amd import workload
    wl = dataclasses.replace(synth.WORKLOADS["tiny-b4"], kv_fill="normal")
    dw = workload.build(wl)
    tok = torch.zeros(4, dtype=torch.int32, device="cuda")
    lp = torch.zeros(4, dtype=torch.float32, device="cuda")
    n = torch.zeros(4, dtype=torch.int32, device="cuda")
    args = (dw.kv, dw.tokens, dw.positions, dw.seq_lens_d, dw.table_d)
    for bad in (0.0, -0.1, 1.5, float("nan")):
        with pytest.raises(hx.HexError):
            dw.engine.decode_step_top_p(*args, 1.0, bad, 1, dw.logits, tok, lp)
    with pytest.raises(hx.HexError):
        dw.engine.decode_step_top_p(*args, 0.0, 0.9, 1, dw.logits, tok, lp)
    with pytest.raises(hx.HexError):                      # the selection needs the stored logits
        dw.engine.decode_step_top_p(*args, 1.0, 0.9, 1, None, tok, lp)
    with pytest.raises(hx.HexError):
        dw.engine.decode_step_top_p(*args, 1.0, 0.9, 1, dw.logits, tok, None)
    with pytest.raises(hx.HexError):                      # sizes are not produced without truncation
        dw.engine.decode_step_top_p(*args, 1.0, 1.0, 1, dw.logits, tok, lp, None, n)
