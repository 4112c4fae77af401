"""Lock-step trajectory parity: the HIP path and the CPU oracle free-run Algorithm 1 from the same seed and the
same synthetic inputs; after every step tokens, normalised log-weights, ESS, resampling flags, ancestors, token
histories, cumulative log p and live KV bytes are compared.

Decisions are discontinuous in the weights, so a mismatch is excused only where the ORACLE says the decision was
ambiguous (two Gumbel keys closer than 1e-6; ESS within 1e-4 of kappa*N; a resampling position within 1e-5 of a
cumulative weight).  An excused event is counted and the device state is overwritten from the oracle; any other
mismatch fails the test.
"""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2602_10273_amd import synth
from paper_2602_10273_amd.harness import Session, to_device_logits

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _resync_hist(s, o, t):
    _, _, par = s.state()
    h = torch.as_tensor(o.hist[:, :t]).cuda()
    pa = torch.as_tensor(par.astype(bool)).cuda()
    s.histA[~pa, :t] = h[~pa]
    s.histB[pa, :t] = h[pa]


def _ambiguous_resample(o, lnw, t):
    """Per prompt: smallest distance between a resampling position and a cumulative weight (oracle quantities)."""
    out = np.full(o.B, np.inf)
    for b in range(o.B):
        w = np.exp(lnw[b * o.N:(b + 1) * o.N])
        C = np.cumsum(w)
        u0 = orc.uniform(orc.random_word(o.seed, t, b, 0, 1))
        p = (u0 + np.arange(o.N)) / o.N
        out[b] = np.abs(C[None, :] - p[:, None]).min()
    return out


def run_lockstep(w, seed, steps, tau=-1.0, table=None, grow_kv=True, kv_seed=3, eos_id=-1, in_place=False,
                 skip_terminated_kv=False, logits_fn=None, fused=False):
    """logits_fn(t) -> (numpy logits for the oracle, device tensor with the same bits): for shapes too large to draw
    on the CPU.  fused: smc_step_resample (one launch) instead of smc_step + smc_ess + smc_resample."""
    from paper_2602_10273_amd import binding as smc
    kv = synth.kv_numpy(w, kv_seed)
    T_max = (steps + 3) // 4 * 4
    s = Session(w.B, w.N, w.V, T_max, w.dtype, w.kappa, seed, kv=kv, eos_id=eos_id)
    if in_place:
        smc.smc_set_ancestor_order(s.ctx, 1)
    if skip_terminated_kv:
        smc.smc_set_kv_skip_terminated(s.ctx, 1)
    o = orc.OracleSMC(w.B, w.N, w.V, T_max, w.kappa, seed, w.dtype, kv=[k.copy() for k in kv], eos_id=eos_id,
                      in_place=in_place, skip_terminated_kv=skip_terminated_kv)
    kv_rng = np.random.default_rng([seed, 99])
    stats = dict(token_ties=0, ess_band=0, pos_band=0, resamples=0, steps=0, max_dw=0.0, max_dess=0.0, done=0,
                 draw_band=0, rows_moved=0)
    for t in range(1, steps + 1):
        x_dev = None
        if logits_fn is not None:
            x, x_dev = logits_fn(t)
        elif table is not None:
            prev = np.zeros(w.R, np.int64) if t == 1 else o.hist[:, t - 2]
            x = synth.logits_numpy(w, t, seed, prev_tokens=prev, table=table)
        else:
            x = synth.logits_numpy(w, t, seed)
        if x_dev is None:
            x_dev = to_device_logits(x, w.dtype)
        a_t, a_p = w.alpha_at(t), w.alpha_at(t - 1)
        want = o.step(x, t, a_t, a_p, tau)
        if fused:
            s.step_resample(x_dev, t, a_t, a_p, tau)
        else:
            s.step(x_dev, t, a_t, a_p, tau)
        got = s.tokens.cpu().numpy()
        mism = got != want["tokens"]
        tie = want["gap"] < 1e-6
        assert not np.any(mism & ~tie), (t, np.nonzero(mism & ~tie)[0][:8])
        dirty = bool(mism.any())
        stats["token_ties"] += int(mism.sum())

        e_ref, lnw_ref = o.ess()
        if fused:                           # the weights were reset inside the launch: only the ESS is there to compare
            e = s.ess.cpu().numpy()
            if not dirty or tau <= 0:
                stats["max_dess"] = max(stats["max_dess"], float(np.abs(e - e_ref).max()))
                assert np.abs(e - e_ref).max() < TOL, t
        else:
            s.compute_ess()
            lnw = s.lognormw.cpu().numpy(); e = s.ess.cpu().numpy()
            if not dirty or tau <= 0:       # with tau = 1/alpha the weights do not depend on the token drawn (Thm 1)
                keep = np.exp(lnw_ref) > 1e-12  # log-weights of particles with no mass left are not compared
                stats["max_dw"] = max(stats["max_dw"], float(np.abs(lnw - lnw_ref)[keep].max()))
                stats["max_dess"] = max(stats["max_dess"], float(np.abs(e - e_ref).max()))
                assert np.abs(lnw - lnw_ref)[keep].max() < TOL, t
                assert np.abs(e - e_ref).max() < TOL, t

        anc_ref, flag_ref, _ = o.resample(t)
        if not fused:
            s.resample(t)
        anc = s.anc.cpu().numpy(); flag = s.resampled.cpu().numpy()
        band = np.abs(e_ref - w.kappa * w.N) < TOL
        assert np.array_equal(flag[~band], flag_ref[~band]), t
        if not np.array_equal(flag, flag_ref):
            stats["ess_band"] += 1; dirty = True
        near = _ambiguous_resample(o, lnw_ref, t) < 1e-5
        for b in range(w.B):
            sl = slice(b * w.N, (b + 1) * w.N)
            if flag[b] == flag_ref[b] and not np.array_equal(anc[sl], anc_ref[sl]):
                assert near[b], (t, b, anc[sl], anc_ref[sl])
                stats["pos_band"] += 1; dirty = True
        stats["resamples"] += int(flag_ref.sum())
        stats["rows_moved"] += int((anc_ref != np.arange(w.R)).sum())

        valid = min(t, w.S) if grow_kv else w.S
        if grow_kv and t <= w.S:            # what the decoder does: position t-1 of every live row is appended
            _, _, par = s.state()
            for ten in range(len(kv)):
                new = synth.f32_to_bf16_bits(kv_rng.standard_normal((w.R, w.H, w.D), dtype=np.float32))
                o.kv[ten][:, :, t - 1, :] = new
                nd = torch.as_tensor(new.view(np.int16)).cuda()
                pa = torch.as_tensor(par.astype(bool)).cuda()
                s.kvA[ten][~pa, :, t - 1, :] = nd[~pa]
                s.kvB[ten][pa, :, t - 1, :] = nd[pa]
        done_before_reindex = o.done.copy()
        if eos_id >= 0 and not dirty:
            assert np.array_equal(s.done(), o.done), t          # termination flags after the step
        o.reindex(anc_ref, flag_ref, valid, t)
        if dirty:                           # follow the oracle's decisions and state
            if eos_id >= 0:
                s.set_done(done_before_reindex)
            s.reindex(valid, t, torch.as_tensor(anc_ref).cuda(), torch.as_tensor(flag_ref).cuda())
            s.set_state(o.logW, o.cumlogp)
            _resync_hist(s, o, t)
        else:
            s.reindex(valid, t)
        logW, cum, _ = s.state()
        assert np.abs(logW - o.logW).max() < TOL and np.abs(cum - o.cumlogp).max() < TOL, t
        assert np.array_equal(s.live_hist()[:, :t], o.hist[:, :t]), t
        if t % 8 == 0 or t == steps:
            ok = o.kv_specified                 # all rows, unless the terminated-ancestor shortcut is on (the oracle says)
            for ten in range(len(kv)):
                assert np.array_equal(s.live_kv(ten)[ok][:, :, :valid], o.kv[ten][ok][:, :, :valid]), (t, ten)
        if eos_id >= 0:
            assert np.array_equal(s.done(), o.done), t          # ... and after they followed their ancestors
        stats["steps"] += 1
    stats["done"] = int(o.done.sum())
    stats["kv_unspecified"] = int((~o.kv_specified).sum())
    if stats["ess_band"] == 0:              # same resampling times on both sides: the estimates of log Z_alpha agree
        assert np.abs(s.log_Zhat() - o.log_Z_estimate()).max() < TOL
    # output of Alg. 1: one particle per prompt from the final weights
    pick_ref = o.final_draw(steps)
    s.final_draw(steps)
    pick = s.choice.cpu().numpy()
    _, lnw_ref = o.ess()
    for b in range(w.B):
        if pick[b] != pick_ref[b]:
            C = np.cumsum(np.exp(lnw_ref[b * w.N:(b + 1) * w.N]))
            u = orc.uniform(orc.random_word(seed, steps, b, 0, 2))
            assert np.abs(C - u).min() < 1e-5, (b, pick[b], pick_ref[b])
            stats["draw_band"] += 1
    s.close()
    return stats


def test_cfg1_tiny_enumerable_full_trajectories():
    w1 = synth.WORKLOADS["cfg1"]
    table = synth.bigram_table(w1.V, w1.sigma, seed=0)
    total = dict(resamples=0, token_ties=0)
    for seed in range(40):
        st = run_lockstep(w1, seed, w1.steps, table=table)
        total["resamples"] += st["resamples"]; total["token_ties"] += st["token_ties"]
    assert total["resamples"] > 3 and total["token_ties"] <= 1
    # many independent copies of the prompt in one batch
    wb = synth.scaled(w1, B=500)
    st = run_lockstep(wb, 1234, w1.steps, table=table)
    assert st["resamples"] > 20


@pytest.mark.parametrize("name,kw,steps", [
    ("cfg2", dict(B=16, N=8, V=8200, layers=2, H=2, S=48, D=64), 48),
    ("cfg3", dict(B=8, N=16, V=6152, layers=1, H=2, S=40, D=128), 40),
    ("cfg4", dict(B=8, N=32, V=4100, layers=1, H=2, S=160, D=32, ramp=128), 160),
    ("cfg5", dict(B=4, N=64, V=9000, layers=1, H=1, S=32, D=64), 32),
])
def test_reduced_workloads_lockstep(name, kw, steps):
    w = synth.scaled(synth.WORKLOADS[name], **kw)
    st = run_lockstep(w, seed=0, steps=steps)
    print(name, st)
    assert st["resamples"] > 0
    assert st["token_ties"] + st["ess_band"] + st["pos_band"] <= 2


def test_eos_absorbing_state_lockstep():
    """Terminated particles: forced EOS, weight kept, flags gathered by ancestor (Alg. 1 'if done'; App. D)."""
    w1 = synth.WORKLOADS["cfg1"]
    table = synth.bigram_table(w1.V, w1.sigma, seed=0)
    st = run_lockstep(synth.scaled(w1, B=400), 77, w1.steps, table=table, eos_id=3)
    assert st["done"] > 100 and st["resamples"] > 10
    # a wider vocabulary with an exponent ramp (the boundary reweight reaches terminated particles too)
    w = synth.scaled(synth.WORKLOADS["cfg4"], B=8, N=16, V=264, layers=1, H=1, S=32, D=32, ramp=16)
    st = run_lockstep(w, seed=2, steps=32, eos_id=5)
    assert st["done"] > 0 and st["kv_unspecified"] == 0          # default: every KV byte follows the gather


def test_eos_lockstep_with_the_terminated_ancestor_shortcut():
    """smc_set_kv_skip_terminated(1): KV rows of terminated ancestors are not moved; the oracle (same option) says which
    rows' bytes are unspecified from then on, every other byte is compared."""
    w1 = synth.WORKLOADS["cfg1"]
    table = synth.bigram_table(w1.V, w1.sigma, seed=0)
    st = run_lockstep(synth.scaled(w1, B=400), 77, w1.steps, table=table, eos_id=3, skip_terminated_kv=True)
    assert st["done"] > 100 and st["resamples"] > 10 and st["kv_unspecified"] > 0
    w = synth.scaled(synth.WORKLOADS["cfg4"], B=8, N=16, V=264, layers=1, H=1, S=32, D=32, ramp=16)
    st = run_lockstep(w, seed=2, steps=32, eos_id=5, skip_terminated_kv=True)
    assert st["done"] > 0


def test_off_optimal_proposal_lockstep():
    """tau != 1/alpha: the increment depends on the sampled token, so token parity feeds the weights."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=6, N=8, V=3000, layers=1, H=1, S=24, D=64, dtype="f32")
    st = run_lockstep(w, seed=4, steps=24, tau=0.4)
    assert st["resamples"] > 0


def test_survivors_in_place_lockstep():
    """Ancestor order 1: the same particle system with every surviving ancestor left in its slot; fewer rows move."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=16, N=8, V=8200, layers=2, H=2, S=48, D=64)
    st0 = run_lockstep(w, seed=0, steps=48)
    st1 = run_lockstep(w, seed=0, steps=48, in_place=True)
    print(st0, st1)
    assert st1["resamples"] > 0 and st1["rows_moved"] < st0["rows_moved"]
    w = synth.scaled(synth.WORKLOADS["cfg5"], B=4, N=64, V=9000, layers=1, H=1, S=32, D=64)
    st = run_lockstep(w, seed=1, steps=32, in_place=True)
    assert st["resamples"] > 0
    w1 = synth.WORKLOADS["cfg1"]
    table = synth.bigram_table(w1.V, w1.sigma, seed=0)
    st = run_lockstep(synth.scaled(w1, B=300), 5, w1.steps, table=table, eos_id=3, in_place=True)
    assert st["resamples"] > 10


def test_long_trajectory_512_steps():
    """The number of decode steps the cfg2 workload names (512), at a reduced vocabulary and cache: no drift."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=4, N=8, V=2056, layers=1, H=1, S=512, D=16)
    st = run_lockstep(w, seed=11, steps=512)
    print(st)
    assert st["resamples"] > 100 and st["token_ties"] + st["ess_band"] + st["pos_band"] <= 4
    assert st["max_dw"] < 1e-4 and st["max_dess"] < 1e-4
