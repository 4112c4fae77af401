"""Pins for the other resampling schemes App. E names (stratified, multinomial, residual): textbook structure,
unbiasedness E[#copies of j] = N w_j, and the whole-method normalising-constant check with each of them."""
import numpy as np
import pytest

from oracle import reference as orc
from oracle.enumerate import enumerate_power_target
from paper_2602_10273_amd import synth

W1 = synth.WORKLOADS["cfg1"]
TABLE = synth.bigram_table(W1.V, W1.sigma, seed=0)
SCHEMES = ["systematic", "stratified", "multinomial", "residual"]


def _u(seed, t, b, i):
    return orc.uniform(orc.random_word(seed, t, b, i, 1))


def test_scheme_zero_is_the_papers_systematic_rule():
    rng = np.random.default_rng(0)
    w = rng.dirichlet(np.full(16, 0.4))
    assert np.array_equal(orc.resample_scheme(w, "systematic", 5, 3, 2), orc.systematic(w, _u(5, 3, 2, 0)))


def test_structure_of_each_scheme():
    rng = np.random.default_rng(1)
    N = 12
    for trial in range(30):
        w = rng.dirichlet(np.full(N, 0.5))
        C = np.cumsum(w)
        seed, t, b = 9, 1 + trial, trial % 3
        us = np.array([_u(seed, t, b, i) for i in range(N)])
        A = orc.resample_scheme(w, "stratified", seed, t, b)
        want = [int(np.argmax(C >= (us[i] + i) / N)) if (C >= (us[i] + i) / N).any() else N - 1 for i in range(N)]
        assert list(A) == want and np.all(np.diff(A) >= 0)            # one draw per stratum ((i)/N, (i+1)/N)
        A = orc.resample_scheme(w, "multinomial", seed, t, b)
        want = [int(np.argmax(C >= us[i])) if (C >= us[i]).any() else N - 1 for i in range(N)]
        assert list(A) == want
        A = orc.resample_scheme(w, "residual", seed, t, b)
        fl = np.floor(N * w).astype(int)
        cnt = np.bincount(A, minlength=N)
        assert np.all(cnt >= fl) and cnt.sum() == N                     # deterministic part
        k = fl.sum()
        assert list(A[:k]) == list(np.repeat(np.arange(N), fl))
        if k < N:
            r = (N * w - fl) / (N - k)
            Cr = np.cumsum(r)
            want = [int(np.argmax(Cr >= us[i])) if (Cr >= us[i]).any() else N - 1 for i in range(N - k)]
            assert list(A[k:]) == want


@pytest.mark.parametrize("scheme", SCHEMES)
def test_each_scheme_is_unbiased(scheme):
    rng = np.random.default_rng(2)
    N = 8
    w = rng.dirichlet(np.full(N, 0.6))
    T = 6000
    tot = np.zeros(N)
    sq = np.zeros(N)
    for t in range(1, T + 1):
        c = np.bincount(orc.resample_scheme(w, scheme, 123, t, 0), minlength=N)
        tot += c; sq += c * c
    mean = tot / T
    var = np.maximum(sq / T - mean ** 2, 1e-12)
    z = (mean - N * w) / np.sqrt(var / T + 1e-12)
    assert np.all(np.abs(z) < 5), (scheme, z)
    if scheme == "multinomial":                                         # counts ~ Binomial(N, w_j)
        assert np.allclose(var, N * w * (1 - w), rtol=0.15)
    if scheme in ("systematic", "stratified", "residual"):              # lower variance than multinomial
        assert np.all(var <= N * w * (1 - w) * 1.1 + 0.02)


@pytest.mark.parametrize("scheme", SCHEMES[1:])
def test_normalising_constant_unbiased_under_each_scheme(scheme):
    _, _, log_Z = enumerate_power_target(TABLE, W1.steps, W1.alpha)
    T, a = W1.steps, W1.alpha
    B = 20000
    w = synth.scaled(W1, B=B)
    o = orc.OracleSMC(B, W1.N, w.V, T, 0.5, 41, "f32", scheme=scheme)
    n_res = 0
    for t in range(1, T + 1):
        prev = np.zeros(w.R, np.int64) if t == 1 else o.hist[:, t - 2]
        o.step(synth.logits_numpy(w, t, 0, prev_tokens=prev, table=TABLE), t, a, a)
        anc, flag, _ = o.resample(t)
        o.reindex(anc, flag, 0, t)
        n_res += int(flag.sum())
    z = np.exp(o.log_Z_estimate() - log_Z)
    se = z.std(ddof=1) / np.sqrt(B)
    assert n_res > B // 20 and abs(z.mean() - 1.0) < 4 * se and se < 0.05


def test_survivors_in_place_is_a_permutation_that_fixes_every_ancestor():
    rng = np.random.default_rng(7)
    for N in (1, 2, 5, 8, 33, 64):
        for _ in range(60):
            A = rng.integers(0, N, N).astype(np.int32)
            if rng.random() < 0.5:
                A = np.sort(A)
            P = orc.survivors_in_place(A)
            assert sorted(P) == sorted(A)                                   # same multiset of ancestors
            for j in np.unique(A):
                assert P[j] == j                                            # every survivor keeps its slot
            assert (P != np.arange(N)).sum() == N - len(np.unique(A))       # the fewest possible slots change owner
            # the copies that move keep the order in which they occur in A
            extra, seen = [], set()
            for a in A:
                if a in seen:
                    extra.append(a)
                seen.add(a)
            assert [P[k] for k in range(N) if P[k] != k] == extra
    assert list(orc.survivors_in_place(np.arange(6, dtype=np.int32))) == list(range(6))
    assert list(orc.survivors_in_place(np.array([3, 3, 3, 3], np.int32))) == [3, 3, 3, 3]
    assert list(orc.survivors_in_place(np.array([0, 0, 2, 2, 2, 5], np.int32))) == [0, 0, 2, 2, 2, 5]
    assert list(orc.survivors_in_place(np.array([1, 1, 1, 4, 4, 4], np.int32))) == [1, 1, 1, 4, 4, 4]
    assert list(orc.survivors_in_place(np.array([2, 2, 3, 3, 3, 3], np.int32))) == [2, 3, 2, 3, 3, 3]


def test_normalising_constant_unbiased_with_survivors_in_place():
    _, _, log_Z = enumerate_power_target(TABLE, W1.steps, W1.alpha)
    T, a = W1.steps, W1.alpha
    B = 20000
    w = synth.scaled(W1, B=B)
    o = orc.OracleSMC(B, W1.N, w.V, T, 0.5, 43, "f32", in_place=True)
    n_res = 0
    for t in range(1, T + 1):
        prev = np.zeros(w.R, np.int64) if t == 1 else o.hist[:, t - 2]
        o.step(synth.logits_numpy(w, t, 0, prev_tokens=prev, table=TABLE), t, a, a)
        anc, flag, _ = o.resample(t)
        for b in np.nonzero(flag)[0][:50]:
            loc = anc[b * W1.N:(b + 1) * W1.N] - b * W1.N
            assert all(loc[j] == j for j in np.unique(loc))
        o.reindex(anc, flag, 0, t)
        n_res += int(flag.sum())
    z = np.exp(o.log_Z_estimate() - log_Z)
    se = z.std(ddof=1) / np.sqrt(B)
    assert n_res > B // 20 and abs(z.mean() - 1.0) < 4 * se and se < 0.05
