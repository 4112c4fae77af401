"""Brute-force evaluation of the power target pi_alpha (Eq. "power") on a tiny enumerable bigram model.

TEST INFRASTRUCTURE.  Every length-T sequence over V tokens is listed, its base log-probability is the sum of
the autoregressive factors (Eq. "base") and pi_alpha(y) = p(y)^alpha / Z_alpha with Z_alpha summed explicitly.
"""
import itertools

import numpy as np
from scipy.special import log_softmax, logsumexp


def enumerate_power_target(table, T, alpha, start_token=0, eos_id=-1):
    """table: [V,V] logits, row = previous token.  Returns (seqs [V^T,T] int, log_pi [V^T], log_Z_alpha).

    eos_id >= 0: EOS is an ordinary token followed by an absorbing state (App. D): after the first EOS the only
    continuation is EOS, with probability 1, so a padded sequence with anything else after EOS has probability 0."""
    table = np.asarray(table, np.float64)
    V = table.shape[0]
    logp_tab = log_softmax(table, axis=1)
    seqs = np.array(list(itertools.product(range(V), repeat=T)), dtype=np.int64)
    prev = np.concatenate([np.full((len(seqs), 1), start_token, np.int64), seqs[:, :-1]], axis=1)
    fac = logp_tab[prev, seqs]
    if eos_id >= 0:
        ended = np.cumsum(prev == eos_id, axis=1) > 0            # an EOS occurred strictly before this position
        fac = np.where(ended, np.where(seqs == eos_id, 0.0, -np.inf), fac)
    logp = fac.sum(axis=1)
    log_Z = logsumexp(alpha * logp)
    with np.errstate(invalid="ignore"):
        log_pi = np.where(np.isfinite(logp), alpha * logp - log_Z, -np.inf)
    return seqs, log_pi, float(log_Z)


def position_marginals(seqs, log_pi, V):
    """marg[t, v] = pi_alpha(y_t = v)."""
    T = seqs.shape[1]
    pi = np.exp(log_pi)
    out = np.zeros((T, V))
    for t in range(T):
        np.add.at(out[t], seqs[:, t], pi)
    return out
