"""Whole-method pin: on the tiny enumerable bigram model every sequence can be listed, so the power target
pi_alpha (Eq. "power") is known exactly.  The oracle's particle system must (i) estimate Z_alpha without
bias for any N and any exponent schedule ending at alpha (Sec. 5.3 / App. B), and (ii) give marginals that
converge to the brute-force ones as N grows."""
import numpy as np
import pytest

from oracle import reference as orc
from oracle.enumerate import enumerate_power_target, position_marginals
from paper_2602_10273_amd import synth

W1 = synth.WORKLOADS["cfg1"]
TABLE = synth.bigram_table(W1.V, W1.sigma, seed=0)


def run_bigram(B, N, T, alphas, seed, kappa=0.5, tau=-1.0):
    """Alg. 1 on B independent copies of the prompt (each its own random stream), bigram logits."""
    w = synth.scaled(W1, B=B, N=N)
    o = orc.OracleSMC(B, N, w.V, T, kappa, seed, "f32")
    n_res = 0
    for t in range(1, T + 1):
        prev = np.zeros(w.R, np.int64) if t == 1 else o.hist[:, t - 2]
        x = synth.logits_numpy(w, t, 0, prev_tokens=prev, table=TABLE)
        o.step(x, t, alphas[t], alphas[t - 1], tau)
        anc, flag, _ = o.resample(t)
        o.reindex(anc, flag, valid_len=0, t=t)
        n_res += int(flag.sum())
    return o, n_res


@pytest.fixture(scope="module")
def exact():
    seqs, log_pi, log_Z = enumerate_power_target(TABLE, W1.steps, W1.alpha)
    return seqs, log_pi, log_Z


def test_enumeration_is_a_distribution(exact):
    seqs, log_pi, log_Z = exact
    assert len(seqs) == 8 ** 6
    assert abs(np.exp(log_pi).sum() - 1) < 1e-12
    assert log_Z < 0                                   # sum_y p(y)^alpha <= 1 for alpha >= 1
    # alpha = 1 is the base model: Z = 1 and pi = p
    _, lp1, lz1 = enumerate_power_target(TABLE, 3, 1.0)
    assert abs(lz1) < 1e-12


@pytest.mark.parametrize("schedule", ["constant", "ramp3", "ramp6", "tau_off"])
def test_normalising_constant_estimate_is_unbiased(exact, schedule):
    _, _, log_Z = exact
    T, a = W1.steps, W1.alpha
    tau = -1.0
    if schedule == "constant":
        alphas = [a] * (T + 1)
    elif schedule == "ramp3":
        alphas = [1.0, 2.0, 3.0, 4.0, 4.0, 4.0, 4.0]
    elif schedule == "ramp6":
        alphas = [1.0 + (a - 1.0) * t / T for t in range(T + 1)]
    else:
        alphas, tau = [a] * (T + 1), 0.5             # a proposal other than the locally optimal one
    B = 20000
    o, n_res = run_bigram(B, W1.N, T, alphas, seed=17, tau=tau)
    assert n_res > B // 20                            # resampling really fires in this test
    z = np.exp(o.log_Z_estimate() - log_Z)            # E[Zhat / Z_alpha] = 1
    se = z.std(ddof=1) / np.sqrt(B)
    assert abs(z.mean() - 1.0) < 4 * se
    assert se < 0.05


def test_dropping_the_boundary_term_breaks_unbiasedness(exact):
    """The check above has teeth: a ramp WITHOUT the stage-boundary reweighting targets something else."""
    _, _, log_Z = exact
    T, a = W1.steps, W1.alpha
    alphas = [1.0, 2.0, 3.0, 4.0, 4.0, 4.0, 4.0]
    B = 20000
    w = synth.scaled(W1, B=B, N=W1.N)
    o = orc.OracleSMC(B, W1.N, w.V, T, 0.5, 17, "f32")
    for t in range(1, T + 1):
        prev = np.zeros(w.R, np.int64) if t == 1 else o.hist[:, t - 2]
        x = synth.logits_numpy(w, t, 0, prev_tokens=prev, table=TABLE)
        o.step(x, t, alphas[t], alphas[t], -1.0)      # alpha_prev := alpha_t suppresses the boundary term
        anc, flag, _ = o.resample(t)
        o.reindex(anc, flag, 0, t)
    z = np.exp(o.log_Z_estimate() - log_Z)
    assert abs(z.mean() - 1.0) > 8 * z.std(ddof=1) / np.sqrt(B)


def test_marginals_converge_with_particle_count(exact):
    seqs, log_pi, _ = exact
    T, V = W1.steps, W1.V
    want = position_marginals(seqs, log_pi, V)
    errs = {}
    for N, B in [(4, 8000), (64, 2000), (1024, 150)]:
        o, _ = run_bigram(B, N, T, [W1.alpha] * (T + 1), seed=5)
        _, lnw = o.ess()
        Wn = np.exp(lnw).reshape(B, N)
        est = np.zeros((T, V))
        for t in range(T):
            tok = o.hist[:, t].reshape(B, N)
            for v in range(V):
                est[t, v] = (Wn * (tok == v)).sum(1).mean()
        errs[N] = np.abs(est - want).max()
    # self-normalised estimates are consistent: bias O(1/N); Monte-Carlo noise here is below ~1e-2
    assert errs[64] < 0.5 * errs[4] + 0.01
    assert errs[1024] < 0.012
    assert errs[4] > errs[1024]


def test_whole_sequence_probabilities(exact):
    seqs, log_pi, _ = exact
    T = W1.steps
    top = np.argsort(-log_pi)[:3]
    B, N = 400, 256
    o, _ = run_bigram(B, N, T, [W1.alpha] * (T + 1), seed=9)
    _, lnw = o.ess()
    Wn = np.exp(lnw).reshape(B, N)
    H = o.hist.reshape(B, N, T)
    for s in top:
        hit = np.all(H == seqs[s][None, None, :], axis=2)
        est = (Wn * hit).sum(1)
        p = np.exp(log_pi[s])
        assert abs(est.mean() - p) < 5 * est.std(ddof=1) / np.sqrt(B) + 0.02 * p
