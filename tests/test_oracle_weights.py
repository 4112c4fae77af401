"""Pins for the oracle's log-softmax, incremental weight (Eq. "inc"), Renyi closed forms (Sec. 5.2),
SIS path weight (Eq. "pathweight") and exponent bridging (Sec. 5.3 / App. B)."""
import mpmath as mp
import numpy as np
import pytest
from scipy.special import log_softmax, logsumexp, softmax

from oracle import reference as orc
from paper_2602_10273_amd import synth


def test_logsumexp_matches_library_and_high_precision():
    rng = np.random.default_rng(0)
    for n, scale in [(1, 1.0), (8, 4.0), (1000, 1.0), (5000, 0.25), (3000, 6.0)]:
        x = rng.standard_normal(n) * 5
        assert abs(orc.logsumexp(x, scale) - logsumexp(scale * x)) < 1e-12
    mp.mp.dps = 40
    x = rng.standard_normal(50) * 30
    ref = mp.log(sum(mp.exp(mp.mpf(float(v)) * 3) for v in x))
    assert abs(orc.logsumexp(x, 3.0) - float(ref)) < 1e-12
    assert abs(orc.logsumexp(x + 7.5, 1.0) - (orc.logsumexp(x, 1.0) + 7.5)) < 1e-12      # shift invariance
    assert orc.logsumexp(np.array([1000.0, 1000.0]), 1.0) == pytest.approx(1000 + np.log(2))  # no overflow


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_row_pass_log_probs_match_library(dtype):
    rng = np.random.default_rng(1)
    x32 = (rng.standard_normal(301) * 3).astype(np.float32)
    stored = synth.f32_to_bf16_bits(x32) if dtype == "bf16" else x32
    x = synth.bf16_bits_to_f32(stored).astype(np.float64) if dtype == "bf16" else x32.astype(np.float64)
    alpha, tau = 4.0, 0.4
    out = orc.vocab_row(stored, dtype, 1 / tau, alpha, seed=5, t=2, r=3)
    y = out["token"]
    assert abs(out["logp"] - log_softmax(x)[y]) < 1e-12
    assert abs(out["logq"] - log_softmax(x / tau)[y]) < 1e-12
    assert abs(out["delta"] - (alpha * log_softmax(x)[y] - log_softmax(x / tau)[y])) < 1e-11
    assert abs(out["logZ1"] - logsumexp(x)) < 1e-12 and abs(out["logZb"] - logsumexp(x / tau)) < 1e-12


def test_T1_increment_is_token_independent_at_tau_equals_one_over_alpha():
    # Thm 1: under q* the weight equals sum_u p(u)^alpha whichever token is drawn.
    rng = np.random.default_rng(2)
    x = (rng.standard_normal(16) * 2).astype(np.float32)
    alpha = 4.0
    want = logsumexp(alpha * log_softmax(x.astype(np.float64)))
    for v in range(16):
        d = orc.vocab_row(x, "f32", alpha, alpha, seed=1, t=1, r=0, forced=v)["delta"]
        assert abs(d - want) < 1e-12
    # and it is NOT token independent for another temperature (guards against ignoring beta)
    ds = [orc.vocab_row(x, "f32", 2.0, alpha, seed=1, t=1, r=0, forced=v)["delta"] for v in range(16)]
    assert np.ptp(ds) > 0.1


def test_T2_mean_of_weight_is_proposal_invariant():
    # Proof of Thm 1, step 1: E_{v~q}[omega(v)] = sum_v p(v)^alpha for any q with full support.
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(12) * 1.5).astype(np.float32)
    alpha = 3.0
    p = softmax(x.astype(np.float64))
    for tau in (1.0, 0.7, 1 / 3.0, 0.2, 2.5):
        q = softmax(x.astype(np.float64) / tau)
        d = np.array([orc.vocab_row(x, "f32", 1 / tau, alpha, 1, 1, 0, forced=v)["delta"] for v in range(12)])
        assert abs((q * np.exp(d)).sum() - (p ** alpha).sum()) < 1e-12


def test_T3_renyi_closed_forms():
    # log Z_t = (1 - alpha) H_alpha(p_t) <= 0 (Eq. "renyiZ"); uniform p gives (1 - alpha) log V.
    for V, alpha in [(8, 4.0), (1000, 2.0), (152064 // 64, 6.0)]:
        d = orc.vocab_row(np.full(V, 1.25, np.float32), "f32", alpha, alpha, 0, 1, 0)["delta"]
        assert abs(d - (1 - alpha) * np.log(V)) < 1e-10
    rng = np.random.default_rng(4)
    for alpha in (1.0, 1.5, 4.0, 6.0):
        x = (rng.standard_normal(500) * 3).astype(np.float32)
        p = softmax(x.astype(np.float64))
        d = orc.vocab_row(x, "f32", alpha, alpha, 0, 1, 0)["delta"]
        assert d <= 1e-13
        if alpha != 1.0:
            H = np.log((p ** alpha).sum()) / (1 - alpha)
            assert abs(d - (1 - alpha) * H) < 1e-10
        else:
            assert abs(d) < 1e-12                   # alpha = 1, tau = 1: base model, weight identically 1
    onehot = np.full(64, -200.0, np.float32); onehot[5] = 50.0
    assert abs(orc.vocab_row(onehot, "f32", 4.0, 4.0, 0, 1, 0)["delta"]) < 1e-12   # zero-entropy limit


def _free_run(w, T, seed, alphas, tau=-1.0, kappa=0.0, logits_seed=0):
    o = orc.OracleSMC(w.B, w.N, w.V, T, kappa, seed, w.dtype)
    deltas, logq = [], np.zeros(w.R)
    for t in range(1, T + 1):
        x = synth.logits_numpy(w, t, logits_seed)
        out = o.step(x, t, alphas[t], alphas[t - 1], tau)
        deltas.append(out["delta"])
        xf = synth.bf16_bits_to_f32(x) if w.dtype == "bf16" else x
        beta = orc.beta_of(alphas[t], tau)
        lq = log_softmax(beta * xf.astype(np.float64), axis=1)
        logq += lq[np.arange(w.R), out["tokens"]]
    return o, np.array(deltas), logq


def test_T4_sis_path_weight():
    # Without resampling log W_T = sum_t log Z_t (Eq. "pathweight"), and for any schedule and proposal
    # log W_T = alpha_T * log p(y_{1:T}) - sum_t log q_t(y_t)  (telescoping of boundary + increment terms).
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=2, N=3, V=257)
    T = 7
    const = [4.0] * (T + 1)
    o, deltas, logq = _free_run(w, T, seed=11, alphas=const)
    assert np.allclose(o.logW, deltas.sum(0), atol=1e-12)
    for t in range(1, T + 1):     # each Delta_t is the row's log sum_v p(v)^alpha
        xf = synth.bf16_bits_to_f32(synth.logits_numpy(w, t, 0)).astype(np.float64)
        assert np.allclose(deltas[t - 1], logsumexp(4.0 * log_softmax(xf, axis=1), axis=1), atol=1e-11)
    assert np.allclose(o.logW, 4.0 * o.cumlogp - logq, atol=1e-10)
    ramp = [1.0, 1.5, 2.0, 2.5, 3.0, 3.5, 4.0, 4.0]
    for tau in (-1.0, 0.5):
        o, _, logq = _free_run(w, T, seed=11, alphas=ramp, tau=tau)
        assert np.allclose(o.logW, ramp[T] * o.cumlogp - logq, atol=1e-10)


def test_T5_constant_schedule_is_plain_smc_and_boundary_term_is_needed():
    w = synth.scaled(synth.WORKLOADS["cfg4"], B=1, N=4, V=129, ramp=0)
    T = 5
    a = [4.0] * (T + 1)
    o1, d1, _ = _free_run(w, T, 3, a)
    # "ramp" whose stages all equal alpha: identical bits to no ramp at all
    o2 = orc.OracleSMC(w.B, w.N, w.V, T, 0.0, 3, w.dtype)
    for t in range(1, T + 1):
        o2.step(synth.logits_numpy(w, t, 0), t, 4.0, 4.0)
    assert np.array_equal(o1.logW, o2.logW) and np.array_equal(o1.hist, o2.hist)
    # with a real ramp the boundary update changes the weights by (alpha_t - alpha_{t-1}) * cumlogp_{t-1}
    ramp = [1.0, 2.0, 3.0, 4.0, 4.0, 4.0]
    o3 = orc.OracleSMC(w.B, w.N, w.V, T, 0.0, 3, w.dtype)
    x1 = synth.logits_numpy(w, 1, 0)
    o3.step(x1, 1, ramp[1], ramp[0])
    before, cum = o3.logW.copy(), o3.cumlogp.copy()
    out = o3.step(synth.logits_numpy(w, 2, 0), 2, ramp[2], ramp[1])
    assert np.allclose(o3.logW - before - out["delta"], (ramp[2] - ramp[1]) * cum, atol=1e-12)
    assert np.abs((ramp[2] - ramp[1]) * cum).max() > 1e-2


def test_alpha_schedule_of_workloads():
    w = synth.WORKLOADS["cfg4"]
    assert w.alpha_at(0) == 1.0 and w.alpha_at(128) == 4.0 and w.alpha_at(500) == 4.0
    assert w.alpha_at(64) == pytest.approx(2.5)
    inc = np.diff([w.alpha_at(t) for t in range(0, 129)])
    assert np.allclose(inc, 3.0 / 128)            # linear schedule alpha^(l) = 1 + (alpha-1) l / L
    assert synth.WORKLOADS["cfg2"].alpha_at(0) == 4.0
