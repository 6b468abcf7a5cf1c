"""Pins of the oracle's sampler and random numbers (CPU only).

Philox4x32-10: the known-answer vectors published with the generator (Random123
distribution, kat_vectors: zero input, all-ones input, and the digits-of-pi input).
Sampler: closed forms (one candidate, uniform logits, a two-point distribution),
limits (tiny temperature, top_k = 1, tiny top_p all give the argmax), and a second,
independent formulation of the kept set (sorted prefix by numpy) on random inputs;
finally the empirical distribution over many draws against the exact probabilities."""
import numpy as np


def test_philox_known_answers(orc):
    assert orc.philox4x32_10((0, 0, 0, 0), (0, 0)) == (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)
    f = 0xffffffff
    assert orc.philox4x32_10((f, f, f, f), (f, f)) == (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)
    assert orc.philox4x32_10((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0)) == \
        (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1)


def test_uniform_is_24_bits_of_the_first_word(orc):
    for seed, step, row in [(0, 0, 0), (12345678901234567, 99, 3), (2 ** 64 - 1, 2 ** 40 + 7, 63)]:
        x0 = orc.philox4x32_10((step & 0xffffffff, step >> 32, row, 0), (seed & 0xffffffff, seed >> 32))[0]
        u = orc.sample_uniform(seed, step, row)
        assert u == (x0 >> 8) / 2.0 ** 24 and 0.0 <= u < 1.0


def test_closed_forms(orc):
    n = 50
    flat = np.zeros(n, dtype=np.float32)
    # equal weights: the draw is floor(u * n) (running sum k/n exceeds u first at k = floor(u n) + 1)
    for u in (0.0, 0.019, 0.5, 0.731, 0.9999):
        assert orc.sample(flat, 1.0, 0, 1.0, u) == int(u * n)
    # two tokens with probabilities 1/4 and 3/4 at temperature 1
    two = np.full(n, -1e9, dtype=np.float32)
    two[7], two[30] = np.log(1.0), np.log(3.0)
    assert orc.sample(two, 1.0, 0, 1.0, 0.2499) == 7 and orc.sample(two, 1.0, 0, 1.0, 0.2501) == 30
    # temperature 1/2 squares the odds: 1/10 and 9/10
    assert orc.sample(two, 0.5, 0, 1.0, 0.0999) == 7 and orc.sample(two, 0.5, 0, 1.0, 0.1001) == 30
    # top_p = 0.7: the 3/4 token alone reaches it, so 7 can no longer be drawn
    assert orc.sample(two, 1.0, 0, 0.7, 0.01) == 30
    # top_p = 0.8 needs both
    assert orc.sample(two, 1.0, 0, 0.8, 0.01) == 7
    # top_k = 1 keeps the maximum only
    assert orc.sample(two, 1.0, 1, 1.0, 0.01) == 30


def test_limits_give_the_argmax(orc):
    rng = np.random.default_rng(1)
    for _ in range(20):
        l = rng.normal(size=300).astype(np.float32)
        best = int(np.argmax(l))
        u = float(rng.random())
        assert orc.sample(l, 1e-4, 0, 1.0, u) == best
        assert orc.sample(l, 1.0, 1, 1.0, u) == best
        assert orc.sample(l, 1.0, 0, 1e-9, u) == best


def kept_set_numpy(l, T, top_k, top_p):
    """Second formulation: stable sort by descending weight, cut by position (top-k) and by
    running mass (top-p), extend both cuts over equal values."""
    s = l.astype(np.float64) / T
    p = np.exp(s - s.max())
    order = np.argsort(-p, kind="stable")
    ps = p[order]
    n = len(p)
    ncand = n
    if 0 < top_k < n:
        ncand = int(np.searchsorted(-ps, -ps[top_k - 1], side="right"))
    keep = ncand
    if top_p < 1.0:
        cum = np.cumsum(ps[:ncand])
        j = int(np.argmax(cum >= top_p * cum[-1]))
        keep = int(np.searchsorted(-ps[:ncand], -ps[j], side="right"))
    kept = np.zeros(n, dtype=bool)
    kept[order[:keep]] = True
    return p, kept


def test_kept_set_and_draw_against_sorted_prefix_formulation(orc):
    rng = np.random.default_rng(2)
    for case in range(60):
        n = int(rng.integers(5, 400))
        l = (rng.normal(size=n) * rng.uniform(0.5, 4)).astype(np.float32)
        if case % 5 == 0:
            l[rng.integers(n, size=n // 3)] = l[0]            # ties, also at the cuts
        T = float(rng.uniform(0.3, 2.0))
        top_k = int(rng.choice([0, 1, 3, 10, n + 5]))
        top_p = float(rng.choice([1.0, 0.95, 0.5, 0.1]))
        p, kept = kept_set_numpy(l, T, top_k, top_p)
        idx = np.flatnonzero(kept)
        cum = np.cumsum(p[idx])
        for u in rng.random(5):
            want = int(idx[min(int(np.searchsorted(cum, u * cum[-1], side="right")), len(idx) - 1)])
            got = orc.sample(l, T, top_k, top_p, float(u))
            if got != want:      # only a draw sitting on a boundary up to rounding may differ
                r = u * cum[-1]
                assert np.min(np.abs(cum - r)) < 1e-9 * cum[-1], (case, got, want)


def test_empirical_distribution(orc):
    l = np.array([0.0, 1.0, 2.0, -1.0, 0.5], dtype=np.float32)
    p = np.exp(l.astype(np.float64))
    p /= p.sum()
    n = 20000
    draws = np.array([orc.sample(l, 1.0, 0, 1.0, orc.sample_uniform(42, step, 0)) for step in range(n)])
    freq = np.bincount(draws, minlength=5) / n
    assert np.abs(freq - p).max() < 4 * np.sqrt(0.25 / n)      # four standard deviations of a proportion
