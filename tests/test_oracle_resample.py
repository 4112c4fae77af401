"""Pins for the oracle's ESS (Eq. "ess"), systematic resampling (Sec. 7) and reindexing (Alg. 1, App. C)."""
from fractions import Fraction

import mpmath as mp
import numpy as np

from oracle import reference as orc


def test_ess_special_cases_and_definition():
    N = 16
    e, lnw = orc.ess(np.full(N, -3.7), 1, N)
    assert abs(e[0] - N) < 1e-12 and np.allclose(np.exp(lnw), 1 / N)
    onehot = np.full(N, -1e4); onehot[3] = 2.0
    assert abs(orc.ess(onehot, 1, N)[0][0] - 1.0) < 1e-12
    rng = np.random.default_rng(0)
    lw = rng.standard_normal(3 * N) * 4
    e, lnw = orc.ess(lw, 3, N)
    e_shift, _ = orc.ess(lw + 123.4, 3, N)                       # invariant to scaling the unnormalised weights
    assert np.allclose(e, e_shift, rtol=1e-12)
    assert np.all(e >= 1 - 1e-12) and np.all(e <= N + 1e-12)
    mp.mp.dps = 40
    for b in range(3):                                            # literal 1 / sum_i W_i^2 in high precision
        wt = [mp.exp(mp.mpf(float(v))) for v in lw[b * N:(b + 1) * N]]
        tot = sum(wt)
        ref = 1 / sum((x / tot) ** 2 for x in wt)
        assert abs(e[b] - float(ref)) < 1e-11 * float(ref)
        assert abs(np.exp(lnw[b * N:(b + 1) * N]).sum() - 1) < 1e-12
    # prompts are independent: per-prompt results do not depend on the batch they sit in
    assert abs(orc.ess(lw[N:2 * N], 1, N)[0][0] - e[1]) == 0


def _systematic_exact(w_frac, u0_frac):
    """The printed rule evaluated in rational arithmetic: p_i=(u0+i-1)/N (1-based), A_i=min{j: sum_{k<=j} w_k >= p_i}."""
    N = len(w_frac)
    A = []
    for i in range(1, N + 1):
        p = (u0_frac + i - 1) / N
        c = Fraction(0)
        for j in range(1, N + 1):
            c += w_frac[j - 1]
            if c >= p:
                A.append(j - 1)
                break
    return A


def test_systematic_matches_rational_evaluation_of_printed_rule():
    rng = np.random.default_rng(1)
    for N in (1, 2, 3, 4, 7):
        for _ in range(40):
            ints = rng.integers(1, 50, size=N)
            wf = [Fraction(int(a), int(ints.sum())) for a in ints]
            u0 = Fraction(int(rng.integers(1, 997)), 997)
            want = _systematic_exact(wf, u0)
            # skip draws that sit within rounding of a boundary in floating point
            cs = np.cumsum([float(x) for x in wf])
            ps = (float(u0) + np.arange(N)) / N
            if np.abs(cs[None, :] - ps[:, None]).min() < 1e-12:
                continue
            got = orc.systematic(np.array([float(x) for x in wf]), float(u0))
            assert list(got) == want


def test_systematic_structure():
    rng = np.random.default_rng(2)
    for N in (4, 8, 32, 64):
        for _ in range(50):
            w = rng.dirichlet(np.full(N, 0.3))
            u0 = rng.uniform()
            A = orc.systematic(w, u0)
            cnt = np.bincount(A, minlength=N)
            assert cnt.sum() == N and np.all(np.diff(A) >= 0)
            assert np.all(cnt >= np.floor(N * w - 1e-9)) and np.all(cnt <= np.ceil(N * w + 1e-9))
        assert list(orc.systematic(np.full(N, 1.0 / N), 0.37)) == list(range(N))      # uniform weights: identity
    one = np.zeros(8); one[5] = 1.0
    assert list(orc.systematic(one, 0.9)) == [5] * 8


def test_systematic_is_unbiased_over_the_offset():
    # E_{u0}[copies of i] = N w_i  (App. E: systematic resampling is unbiased)
    rng = np.random.default_rng(3)
    N = 8
    w = rng.dirichlet(np.full(N, 0.5))
    G = 20000
    tot = np.zeros(N)
    for k in range(G):
        tot += np.bincount(orc.systematic(w, (k + 0.5) / G), minlength=N)
    assert np.allclose(tot / G, N * w, atol=2.0 / G * N)


def test_resample_trigger_offset_and_reset():
    B, N, seed, t = 5, 8, 2024, 7
    rng = np.random.default_rng(4)
    logW = rng.standard_normal(B * N)
    logW[0:N] = 0.0                              # ESS = N: never resamples for kappa < 1
    logW[N:2 * N] = [0, -50, -50, -50, -50, -50, -50, -50]      # ESS ~ 1: resamples
    anc, flag, e, lw_after = orc.resample(logW, B, N, 0.5, seed, t)
    e_ref, lnw = orc.ess(logW, B, N)
    assert np.array_equal(e, e_ref)
    assert np.array_equal(flag, (e_ref < 0.5 * N).astype(np.int32))      # strict '<' (Alg. 1)
    assert flag[0] == 0 and flag[1] == 1
    for b in range(B):
        sl = slice(b * N, (b + 1) * N)
        if flag[b]:
            u0 = orc.uniform(orc.random_word(seed, t, b, 0, 1))          # offset from the resampling domain
            want = b * N + orc.systematic(np.exp(lnw[sl]), u0)
            assert np.array_equal(anc[sl], want)
            assert np.all(lw_after[sl] == 0.0)                            # weights reset to 1
        else:
            assert np.array_equal(anc[sl], np.arange(b * N, (b + 1) * N))
            assert np.array_equal(lw_after[sl], logW[sl])
    assert np.array_equal(anc[N:2 * N], np.full(N, N))                    # all mass on particle 0 of prompt 1
    # threshold is strict: ESS exactly equal to kappa*N does not resample
    two = np.array([0.0, 0.0, -np.inf, -np.inf])                          # ESS = 2 exactly, N = 4, kappa = 0.5
    _, f, e2, _ = orc.resample(two, 1, 4, 0.5, seed, t)
    assert e2[0] == 2.0 and f[0] == 0


def test_gather_kv_and_state():
    rng = np.random.default_rng(5)
    B, N, H, S, D = 3, 4, 2, 5, 8
    R = B * N
    src = rng.integers(0, 65535, size=(R, H, S, D)).astype(np.uint16)
    anc = np.arange(R, dtype=np.int32)
    anc[0:4] = [1, 1, 3, 3]
    anc[8:12] = [11, 10, 9, 8]
    flag = np.array([1, 0, 1], np.int32)
    dst0 = np.full_like(src, 0xAAAA)
    dst = orc.gather_kv(src, anc, flag, N, S, dst0.copy())
    for k in range(R):
        if flag[k // N]:
            assert np.array_equal(dst[k], src[anc[k]])
        else:
            assert np.all(dst[k] == 0xAAAA)                   # prompts that did not resample are not touched
    part = orc.gather_kv(src, anc, flag, N, 3, dst0.copy())   # only the first valid_len positions of each head
    for k in (0, 1, 2, 3, 8, 9, 10, 11):
        assert np.array_equal(part[k][:, :3], src[anc[k]][:, :3]) and np.all(part[k][:, 3:] == 0xAAAA)
    # permutation ancestors preserve the multiset of rows; identity ancestors reproduce the source
    assert sorted(map(bytes, dst[8:12])) == sorted(map(bytes, src[8:12]))
    ident = orc.gather_kv(src, np.arange(R, dtype=np.int32), np.ones(B, np.int32), N, S)
    assert np.array_equal(ident, src)

    o = orc.OracleSMC(B, N, 16, 6, 0.5, 1, "f32", kv=[src.copy(), src[::-1].copy()])
    o.hist[:] = rng.integers(0, 16, size=(R, 6)); o.cumlogp[:] = rng.standard_normal(R)
    h0, c0, kv1 = o.hist.copy(), o.cumlogp.copy(), o.kv[1].copy()
    o.reindex(anc, flag, valid_len=S, t=4)
    for k in range(R):
        a = anc[k] if flag[k // N] else k
        assert np.array_equal(o.hist[k, :4], h0[a, :4]) and o.cumlogp[k] == c0[a]
        assert np.array_equal(o.kv[0][k], src[a]) and np.array_equal(o.kv[1][k], kv1[a])
    assert np.array_equal(o.hist[:, 4:], h0[:, 4:])           # columns beyond t are left alone
