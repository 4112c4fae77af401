"""Property-based checks of the CPU oracle (hypothesis): statements that hold for every input, drawn at random.

Each property is one the paper or the mathematics fixes -- the weight identity at tau = 1/alpha (Thm 1), the mean of the
incremental weight under any proposal (proof of Thm 1, step 1), the range and invariances of ESS (Eq. "ess"), the
copy counts of systematic resampling (Sec. 7), the row gather (Alg. 1 "reorder"; App. C) -- so a slip in the oracle
that the fixed-seed pins happen to miss still has to survive these."""
import numpy as np
from hypothesis import given, settings, strategies as st
from scipy.special import logsumexp as sp_lse

from oracle import reference as orc

SET = settings(max_examples=60, deadline=None)

logit_rows = st.integers(2, 40).flatmap(lambda V: st.lists(
    st.floats(-30.0, 30.0, allow_nan=False, width=32), min_size=V, max_size=V))
alphas = st.floats(1.0, 8.0, allow_nan=False)


@SET
@given(logit_rows, alphas, st.integers(0, 2 ** 40), st.integers(1, 1000), st.integers(0, 5000))
def test_weight_identity_and_normalisation(x, alpha, seed, t, r):
    x = np.asarray(x, np.float32)
    V = x.size
    res = orc.vocab_row(x, "f32", alpha, alpha, seed, t, r)
    assert 0 <= res["token"] < V and res["second"] != res["token"]
    assert abs(res["logZ1"] - sp_lse(x.astype(np.float64))) < 1e-9
    assert abs(res["logZb"] - sp_lse(alpha * x.astype(np.float64))) < 1e-9
    assert res["logp"] <= 1e-12 and res["logq"] <= 1e-12
    # Thm 1: at tau = 1/alpha the increment is log sum_v p(v)^alpha whatever token was drawn
    want = res["logZb"] - alpha * res["logZ1"]
    for forced in {0, V - 1, res["token"]}:
        assert abs(orc.vocab_row(x, "f32", alpha, alpha, seed, t, r, forced=forced)["delta"] - want) < 1e-9
    assert want <= 1e-12                                     # (1 - alpha) H_alpha(p) <= 0 for alpha >= 1


@SET
@given(logit_rows, alphas, st.floats(0.25, 8.0, allow_nan=False), st.integers(0, 2 ** 40))
def test_mean_incremental_weight_is_proposal_invariant(x, alpha, beta, seed):
    """E_{v ~ q}[p(v)^alpha / q(v)] = sum_v p(v)^alpha for any proposal q = softmax(beta * logits)."""
    x = np.asarray(x, np.float32)
    V = x.size
    rows = [orc.vocab_row(x, "f32", beta, alpha, seed, 1, 0, forced=v) for v in range(V)]
    logq = np.array([r["logq"] for r in rows]); delta = np.array([r["delta"] for r in rows])
    assert abs(sp_lse(logq)) < 1e-9                          # q is a distribution
    lhs = sp_lse(logq + delta)                               # log sum_v q(v) * w(v)
    rhs = sp_lse(alpha * (x.astype(np.float64) - sp_lse(x.astype(np.float64))))        # log sum_v p(v)^alpha
    assert abs(lhs - rhs) < 1e-8


weights = st.integers(1, 24).flatmap(lambda N: st.lists(st.floats(-20.0, 5.0, allow_nan=False), min_size=N, max_size=N))


@SET
@given(weights, st.floats(-50.0, 50.0, allow_nan=False))
def test_ess_range_and_shift_invariance(lw, shift):
    lw = np.asarray(lw, np.float64)
    N = lw.size
    e, lnw = orc.ess(lw, 1, N)
    assert 1.0 - 1e-9 <= e[0] <= N + 1e-9
    assert abs(sp_lse(lnw)) < 1e-9
    e2, _ = orc.ess(lw + shift, 1, N)
    assert abs(e2[0] - e[0]) < 1e-7 * N
    W = np.exp(lnw)
    assert abs(e[0] - 1.0 / np.sum(W * W)) < 1e-7 * N


@SET
@given(weights, st.floats(0.0, 1.0, exclude_max=True, allow_nan=False))
def test_systematic_copy_counts(lw, u0):
    lw = np.asarray(lw, np.float64)
    N = lw.size
    w = np.exp(lw - sp_lse(lw))
    A = orc.systematic(w, u0)
    assert np.all(np.diff(A) >= 0) and A.min() >= 0 and A.max() < N
    counts = np.bincount(A, minlength=N)
    assert counts.sum() == N
    slack = 1e-9 * N
    assert np.all(counts >= np.floor(N * w - slack)) and np.all(counts <= np.ceil(N * w + slack))
    P = orc.survivors_in_place(A)
    assert np.array_equal(np.sort(P), A)                     # a permutation of the same ancestors
    for a in np.unique(A):
        assert P[a] == a                                     # every distinct ancestor keeps its own slot
    assert int(np.sum(P != np.arange(N))) == N - np.unique(A).size


@SET
@given(st.integers(1, 3), st.integers(1, 6), st.integers(1, 3), st.integers(1, 5), st.integers(0, 2 ** 31), st.data())
def test_gather_is_the_indexed_copy(B, N, H, S, seed, data):
    rng = np.random.default_rng(seed)
    D, R = 2, B * N
    src = rng.integers(0, 65536, (R, H, S, D), dtype=np.uint16)
    dst0 = rng.integers(0, 65536, (R, H, S, D), dtype=np.uint16)
    anc = np.concatenate([b * N + rng.integers(0, N, N) for b in range(B)]).astype(np.int32)
    flag = rng.integers(0, 2, B).astype(np.int32)
    valid = data.draw(st.integers(0, S))
    dst = orc.gather_kv(src, anc, flag, N, valid, dst0.copy())
    for k in range(R):
        if flag[k // N]:
            assert np.array_equal(dst[k, :, :valid], src[anc[k], :, :valid])
            assert np.array_equal(dst[k, :, valid:], dst0[k, :, valid:])
        else:
            assert np.array_equal(dst[k], dst0[k])
