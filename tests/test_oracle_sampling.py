"""Pins of the oracle's sampler: the counter-based generator against its published known-answer vectors,
the draw against the distribution it must follow and against library log-softmax, and its limits."""
import os

import numpy as np
import scipy.special
import scipy.stats

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def test_philox_known_answers():
    n = 0
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        assert len(w) == 10
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in out] == w[6:10], line
        n += 1
    assert n == 3


def test_philox_is_a_bijection_of_the_counter_on_a_sample():
    """Distinct counters give distinct blocks (the round function is invertible); the key changes the stream."""
    key = [123, 456]
    seen = {tuple(int(v) for v in oracle.philox4x32_10([i, 7, 9, 0], key)) for i in range(2000)}
    assert len(seen) == 2000
    assert not np.array_equal(oracle.philox4x32_10([1, 2, 3, 4], key), oracle.philox4x32_10([1, 2, 3, 4], [123, 457]))


def test_uniform_is_strictly_inside_the_unit_interval():
    """23 random bits + one half: every value is exact in fp32 and neither 0 nor 1 can occur (24 bits would
    round the top value to 1.0 and make the Gumbel term infinite)."""
    assert oracle.uniform_open(0) == 0.5 / 2 ** 23
    assert oracle.uniform_open(0xFFFFFFFF) == 1.0 - 0.5 / 2 ** 23
    assert 0.0 < oracle.uniform_open(0) and oracle.uniform_open(0xFFFFFFFF) < 1.0
    assert oracle.uniform_open(0x80000000) == 0.5 + 0.5 / 2 ** 23


def _draw(logits, temperature, n, seed=99, pos=5):
    B = n
    x = np.broadcast_to(np.asarray(logits, dtype=np.float32), (B, len(logits)))
    return oracle.sample(x, temperature, seed, np.arange(B), np.full(B, pos))


def test_draws_follow_softmax_of_scaled_logits():
    """Chi-square of 60 000 independent rows (row id enters the counter) against softmax(logits / T); a wrong
    Gumbel sign, a temperature applied the wrong way round or correlated words all fail it."""
    logits = np.array([1.0, 0.2, -0.7, 2.1, 0.0, -1.5, 0.9], dtype=np.float32)
    for temperature in (1.0, 0.5, 2.0):
        tok, lp, _ = _draw(logits, temperature, 60000)
        p = scipy.special.softmax(logits.astype(np.float64) / temperature)
        counts = np.bincount(tok, minlength=len(logits))
        chi2 = float(((counts - 60000 * p) ** 2 / (60000 * p)).sum())
        assert chi2 < scipy.stats.chi2.ppf(0.9999, len(logits) - 1), (temperature, chi2)
        # a distribution that ignores the temperature is rejected by the same test (T != 1)
        if temperature != 1.0:
            q = scipy.special.softmax(logits.astype(np.float64))
            chi2_wrong = float(((counts - 60000 * q) ** 2 / (60000 * q)).sum())
            assert chi2_wrong > 200, chi2_wrong
        # the log-probability is log-softmax at the drawn token (library routine, fp64)
        ref = scipy.special.log_softmax(logits.astype(np.float64) * float(np.float32(1.0) / np.float32(temperature)))
        assert np.abs(lp - ref[tok]).max() < 2e-6


def test_words_of_one_block_and_neighbouring_positions_are_not_reused():
    """Equal logits: every entry equally likely, also within a block of four and across positions."""
    V = 8
    tok_a, _, _ = _draw(np.zeros(V), 1.0, 40000, pos=3)
    tok_b, _, _ = _draw(np.zeros(V), 1.0, 40000, pos=4)
    for tok in (tok_a, tok_b):
        counts = np.bincount(tok, minlength=V)
        chi2 = float(((counts - 5000.0) ** 2 / 5000.0).sum())
        assert chi2 < scipy.stats.chi2.ppf(0.9999, V - 1), chi2
    assert (tok_a == tok_b).mean() < 0.15           # independent streams agree 1/8 of the time


def test_low_temperature_limit_is_the_argmax_and_logprob_tends_to_zero():
    rng = np.random.default_rng(3)
    x = rng.normal(0, 1, size=(50, 300)).astype(np.float32)
    tok, lp, _ = oracle.sample(x, 1e-3, 7, np.arange(50), np.arange(50))
    assert np.array_equal(tok, np.argmax(x, axis=1))
    assert np.all(lp <= 0) and np.all(lp > -1e-3)


def test_draw_depends_on_seed_row_and_position_only():
    rng = np.random.default_rng(4)
    x = rng.normal(0, 1, size=(1, 1000)).astype(np.float32)
    base = oracle.sample(x, 1.0, 11, [5], [77])
    again = oracle.sample(x.copy(), 1.0, 11, [5], [77])
    assert base[0][0] == again[0][0] and base[1][0] == again[1][0]
    others = {int(oracle.sample(x, 1.0, s, [r], [p])[0][0]) for s, r, p in ((12, 5, 77), (11, 6, 77), (11, 5, 78), (2 ** 40 + 11, 5, 77))}
    assert len(others | {int(base[0][0])}) >= 4      # 1000-way draws: four changed inputs give (almost surely) new tokens


def test_gap_is_best_minus_runner_up_of_the_perturbed_scores():
    """Recompute the perturbed scores with numpy from the generator's words."""
    rng = np.random.default_rng(5)
    V, seed, row, pos, T = 37, 2 ** 33 + 5, 3, 900, 0.8
    x = rng.normal(0, 2, size=V).astype(np.float32)
    tok, lp, gap = oracle.sample(x, T, seed, [row], [pos])
    y = np.empty(V, dtype=np.float32)
    inv_t = np.float32(1.0) / np.float32(T)
    for i in range(V):
        word = int(oracle.philox4x32_10([i // 4, row, pos, 0x53414D50], [seed & 0xFFFFFFFF, seed >> 32])[i % 4])
        u = np.float32((np.float32(word >> 9) + np.float32(0.5)) * np.float32(2.0 ** -23))
        y[i] = x[i] * inv_t - np.log(-np.log(u, dtype=np.float32), dtype=np.float32)
    order = np.argsort(-y, kind="stable")
    assert int(tok[0]) == int(order[0])
    assert abs(float(gap[0]) - float(y[order[0]] - y[order[1]])) < 1e-5
