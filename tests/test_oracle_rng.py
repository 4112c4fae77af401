"""Pins for the oracle's random stream: Philox4x32-10, the uniform mapping, the Gumbel variate, Gumbel-max.

The paper does not say how y ~ q_t is drawn (Alg. 1, "sample"); the reading is Gumbel-max with one Philox
word per vocabulary entry.  What pins it: published known-answer vectors, high-precision evaluation of the
closed form, and the distributional identity argmax_v(beta*l_v + g_v) ~ softmax(beta*l).
"""
import os

import mpmath as mp
import numpy as np
import pytest
from scipy import stats
from scipy.special import softmax

from oracle import reference as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert orc.philox4x32_10(ctr, key) == out


def test_philox_is_a_bijection_on_counters_sample():
    # distinct counters under one key give distinct blocks (Philox is a keyed permutation of the counter space)
    seen = set()
    for c in range(2000):
        seen.add(tuple(orc.philox4x32_10([c, 0, 0, 0], [5, 6])))
    assert len(seen) == 2000


def test_random_word_layout():
    # word v of row r at step t: block counter (v//4, r, t, domain), word v%4, key = (seed lo, seed hi)
    seed = 0x1234_5678_9ABC_DEF0
    for (t, r, v, d) in [(1, 0, 0, 0), (3, 17, 5, 0), (9, 2, 152063, 0), (4, 3, 0, 1)]:
        blk = orc.philox4x32_10([v >> 2, r, t, d], [seed & 0xFFFFFFFF, seed >> 32])
        assert orc.random_word(seed, t, r, v, d) == blk[v & 3]
    # changing any coordinate changes the word
    base = orc.random_word(seed, 1, 1, 1, 0)
    assert len({base, orc.random_word(seed + 1, 1, 1, 1, 0), orc.random_word(seed, 2, 1, 1, 0),
                orc.random_word(seed, 1, 2, 1, 0), orc.random_word(seed, 1, 1, 2, 0),
                orc.random_word(seed, 1, 1, 1, 1)}) == 6


def test_random_words_uniform_and_uncorrelated():
    n = 200_000
    x = np.array([orc.random_word(42, 1, 0, v) for v in range(n)], dtype=np.float64) / 2.0**32
    counts, _ = np.histogram(x, bins=64, range=(0, 1))
    chi2 = ((counts - n / 64) ** 2 / (n / 64)).sum()
    assert chi2 < stats.chi2.ppf(1 - 1e-6, 63)
    lag1 = np.corrcoef(x[:-1], x[1:])[0, 1]
    assert abs(lag1) < 5 / np.sqrt(n)


def test_uniform_mapping_open_interval():
    assert orc.uniform(0) == 0.5 * 2.0**-32
    assert orc.uniform(0xFFFFFFFF) == 1.0 - 0.5 * 2.0**-32
    assert 0.0 < orc.uniform(0) < orc.uniform(1) < orc.uniform(0xFFFFFFFF) < 1.0


@pytest.mark.parametrize("x", [0, 1, 2, 1000, 0x7FFFFFFF, 0x80000000, 0x80000001, 0xC0000000,
                               0xFFFF0000, 0xFFFFFFF0, 0xFFFFFFFE, 0xFFFFFFFF, 123456789, 3141592653])
def test_gumbel_matches_high_precision_closed_form(x):
    mp.mp.dps = 50
    u = (mp.mpf(x) + mp.mpf("0.5")) / mp.mpf(2) ** 32
    g = -mp.log(-mp.log(u))
    assert abs(orc.gumbel(x) - float(g)) <= 4e-15 * max(1.0, abs(float(g)))


def test_gumbel_range_and_monotone():
    gmin, gmax = orc.gumbel(0), orc.gumbel(0xFFFFFFFF)
    # u_min = 2^-33 gives g = -log(33 log 2); u_max = 1 - 2^-33 gives g = 33 log 2 up to O(2^-34)
    assert abs(gmin - (-np.log(33 * np.log(2)))) < 1e-12
    assert abs(gmax - 33 * np.log(2)) < 1e-9
    xs = np.unique(np.concatenate([np.arange(0, 64), np.linspace(0, 2**32 - 1, 4001).astype(np.uint64),
                                   np.arange(2**31 - 32, 2**31 + 32), np.arange(2**32 - 64, 2**32)]))
    g = np.array([orc.gumbel(int(x)) for x in xs])
    assert np.all(np.diff(g) > 0)          # also across the u = 1/2 branch switch


def test_gumbel_max_samples_the_tempered_softmax():
    # argmax_v(beta*l_v + g_v) is distributed as softmax(beta*l) (Cor. 1: the proposal softmax(l/tau)).
    V, beta, n = 8, 1.7, 60_000
    logits = np.array([0.3, -1.2, 2.0, 0.0, 1.1, -0.4, 0.9, -2.5], np.float32)
    q = softmax(beta * logits.astype(np.float64))
    counts = np.zeros(V)
    for r in range(n):
        counts[orc.vocab_row(logits, "f32", beta, 1.0, seed=777, t=1 + (r % 3), r=r)["token"]] += 1
    chi2 = ((counts - n * q) ** 2 / (n * q)).sum()
    assert chi2 < stats.chi2.ppf(1 - 1e-5, V - 1)
    # a transposed sign or a missing beta would fail: compare against the wrong temperatures
    for wrong in (softmax(logits.astype(np.float64)), softmax(-beta * logits.astype(np.float64))):
        assert ((counts - n * wrong) ** 2 / (n * wrong)).sum() > 10 * stats.chi2.ppf(1 - 1e-5, V - 1)


def test_argmax_key_is_reproducible_from_parts():
    # token and gap reported by the row pass agree with keys rebuilt from gumbel() and random_word()
    rng = np.random.default_rng(3)
    logits = rng.standard_normal(37).astype(np.float32) * 2
    beta, seed, t, r = 2.5, 99, 4, 6
    keys = np.array([beta * float(logits[v]) + orc.gumbel(orc.random_word(seed, t, r, v)) for v in range(37)])
    out = orc.vocab_row(logits, "f32", beta, 2.5, seed, t, r)
    order = np.argsort(-keys, kind="stable")
    assert out["token"] == order[0] and out["second"] == order[1]
    assert abs(out["gap"] - (keys[order[0]] - keys[order[1]])) < 1e-15
