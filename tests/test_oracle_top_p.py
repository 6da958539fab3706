"""Pins of the oracle's nucleus (top-p) sampler: kept-set sizes worked by hand on a four-entry distribution, the
limits top_p -> 0 and top_p -> 1, ties at the cut, the draw against the renormalised distribution (chi-square) and
the log-probability against a float64 recomputation from a library sort."""
import numpy as np
import scipy.special
import scipy.stats

import oracle


def _rows(logits, n):
    return np.broadcast_to(np.asarray(logits, dtype=np.float32), (n, len(logits)))


def test_kept_set_sizes_of_a_hand_worked_distribution():
    """p = (0.5, 0.3, 0.15, 0.05) given in scrambled order: running masses 0.5, 0.8, 0.95, 1.0, so top_p = 0.4,
    0.75, 0.85, 0.96 keep 1, 2, 3, 4 entries; a prefix rule that stops one entry early or late, or that orders
    ascending, fails."""
    p = np.array([0.15, 0.5, 0.05, 0.3])
    logits = np.log(p).astype(np.float32) + 3.0          # softmax is shift invariant
    for top_p, size in ((0.4, 1), (0.75, 2), (0.85, 3), (0.96, 4)):
        _, _, n, margin, _ = oracle.sample_top_p(_rows(logits, 1), 1.0, top_p, 1, [0], [0])
        assert n[0] == size, (top_p, n)
        assert margin[0] > 0.009
    # the margin is the distance to the nearer deciding mass: top_p = 0.79 sits 0.01 below 0.8
    _, _, n, margin, _ = oracle.sample_top_p(_rows(logits, 1), 1.0, 0.79, 1, [0], [0])
    assert n[0] == 2 and abs(margin[0] - 0.01) < 1e-6


def test_temperature_is_applied_before_the_cut():
    """At T = 0.5 the same logits give p proportional to (0.25, 0.09, 0.0225, 0.0025): the top entry alone holds
    0.685 of the mass, so top_p = 0.6 keeps one entry where T = 1 keeps two."""
    logits = np.log(np.array([0.5, 0.3, 0.15, 0.05])).astype(np.float32)
    assert oracle.sample_top_p(_rows(logits, 1), 1.0, 0.6, 1, [0], [0])[2][0] == 2
    assert oracle.sample_top_p(_rows(logits, 1), 0.5, 0.6, 1, [0], [0])[2][0] == 1


def test_small_top_p_is_greedy_with_certainty():
    rng = np.random.default_rng(5)
    x = rng.normal(0, 1.5, size=(50, 300)).astype(np.float32)
    tok, lp, n, _, _ = oracle.sample_top_p(x, 0.8, 1e-6, 77, np.arange(50), np.arange(50))
    assert np.array_equal(tok, x.argmax(axis=1))
    assert np.all(n == 1) and np.all(lp == 0.0)


def test_top_p_near_one_is_the_plain_sampler():
    """With every entry kept the draw and its log-probability are those of the temperature sampler (same noise)."""
    rng = np.random.default_rng(6)
    x = rng.normal(0, 1.0, size=(40, 64)).astype(np.float32)
    rows, pos = np.arange(40) + 3, np.arange(40) * 7
    tok, lp, n, _, _ = oracle.sample_top_p(x, 1.3, 0.99999994, 1234, rows, pos)
    tok0, lp0, _ = oracle.sample(x, 1.3, 1234, rows, pos)
    assert np.all(n == 64)
    assert np.array_equal(tok, tok0)
    assert np.allclose(lp, lp0, atol=1e-6)


def test_entries_tied_with_the_last_kept_one_are_kept():
    logits = np.array([0.0, -10.0, 0.0, 0.0], dtype=np.float32)
    tok, lp, n, _, _ = oracle.sample_top_p(_rows(logits, 3000), 1.0, 0.2, 9, np.arange(3000), np.zeros(3000))
    assert np.all(n == 3)
    assert set(np.unique(tok)) == {0, 2, 3}
    assert np.allclose(lp, np.log(1.0 / 3.0), atol=1e-6)
    counts = np.bincount(tok, minlength=4)[[0, 2, 3]]
    assert float(((counts - 1000.0) ** 2 / 1000.0).sum()) < scipy.stats.chi2.ppf(0.9999, 2)


def test_draws_follow_the_renormalised_kept_set():
    """40 000 independent rows: nothing outside the kept set is ever drawn and the kept entries appear with
    p_i / mass (chi-square); drawing from the untruncated softmax, or truncating without renormalising the
    reported log-probability, fails."""
    logits = np.array([1.0, 0.2, -0.7, 2.1, 0.0, -1.5, 0.9, -3.0], dtype=np.float32)
    temperature, top_p, N = 0.9, 0.8, 40000
    p = scipy.special.softmax(logits.astype(np.float64) / temperature)
    order = np.argsort(-p, kind="stable")
    size = int(np.searchsorted(np.cumsum(p[order]), top_p) + 1)
    kept = order[:size]
    assert 1 < size < len(logits)
    tok, lp, n, _, _ = oracle.sample_top_p(_rows(logits, N), temperature, top_p, 4242, np.arange(N), np.full(N, 11))
    assert np.all(n == size)
    assert set(np.unique(tok)) <= set(int(k) for k in kept)
    q = p[kept] / p[kept].sum()
    counts = np.bincount(tok, minlength=len(logits))[kept]
    chi2 = float(((counts - N * q) ** 2 / (N * q)).sum())
    assert chi2 < scipy.stats.chi2.ppf(0.9999, size - 1), chi2
    full = p[kept]                                        # the untruncated probabilities do not fit
    assert float(((counts - N * full) ** 2 / (N * full)).sum()) > scipy.stats.chi2.ppf(0.9999, size - 1)
    for k, qk in zip(kept, q):
        assert np.allclose(lp[tok == k], np.log(qk), atol=2e-6)


def test_kept_set_and_logprob_against_a_library_sort_in_float64():
    """Vocabulary-sized rows: size of the kept set and log-probability of the drawn token recomputed with
    numpy's sort and cumulative sum in float64 (rows whose deciding mass is within 1e-9 of top_p are skipped:
    none occur with these seeds)."""
    rng = np.random.default_rng(8)
    V, B = 20000, 6
    x = rng.normal(0, 1.2, size=(B, V)).astype(np.float32)
    for temperature, top_p in ((1.0, 0.9), (0.7, 0.5), (1.5, 0.95)):
        tok, lp, n, margin, _ = oracle.sample_top_p(x, temperature, top_p, 31, np.arange(B), np.arange(B) + 100)
        z = (x * np.float32(1.0 / np.float32(temperature))).astype(np.float32).astype(np.float64)
        for b in range(B):
            assert margin[b] > 1e-9
            p = scipy.special.softmax(z[b])
            srt = np.sort(p)[::-1]
            size = int(np.searchsorted(np.cumsum(srt), top_p) + 1)
            assert n[b] == size, (b, n[b], size)
            thr = srt[size - 1]
            assert p[tok[b]] >= thr
            assert abs(lp[b] - np.log(p[tok[b]] / p[p >= thr].sum())) < 2e-6
