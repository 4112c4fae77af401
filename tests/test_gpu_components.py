"""Component parity, HIP path vs CPU oracle, through the C ABI (needs an MI355X).

Bars: tokens and ancestors bit-exact (a token may differ only where the oracle's two best Gumbel keys are closer
than 1e-6; such rows are counted and must be rare), reindexed bytes bit-exact, log-weights / ESS within 1e-4 abs.
"""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2602_10273_amd import binding as smc
from paper_2602_10273_amd import synth
from paper_2602_10273_amd.harness import Session, to_device_logits

pytestmark = pytest.mark.gpu

TOL = 1e-4
NEAR_TIE = 1e-6


def check_step(w, seed, t, alpha_t, alpha_prev, tau, n_split=0, dense=0, logits=None, stride_pad=0, wg_waves=0):
    from paper_2602_10273_amd import binding as smc
    x = synth.logits_numpy(w, t, seed) if logits is None else logits
    if stride_pad:
        # NaN (bf16 bits 0x7FC0 / float NaN) behind every row: nothing past V may be read
        pad = np.full((w.R, stride_pad), 0x7FC0 if x.dtype == np.uint16 else np.nan, x.dtype)
        xs = np.concatenate([x, pad], axis=1)
    else:
        xs = x
    o = orc.OracleSMC(w.B, w.N, w.V, 8, w.kappa, seed, w.dtype)
    rng = np.random.default_rng(seed + 1)
    o.logW[:] = rng.standard_normal(w.R); o.cumlogp[:] = -rng.random(w.R) * 5
    s = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, seed)
    s.set_state(o.logW, o.cumlogp)
    smc.smc_set_tuning(s.ctx, n_split, dense, wg_waves)
    want = o.step(xs, t, alpha_t, alpha_prev, tau, row_stride=xs.shape[1])
    xd = to_device_logits(xs, w.dtype)
    s.step(xd, t, alpha_t, alpha_prev, tau)
    got = s.tokens.cpu().numpy()
    logW, cum, _ = s.state()
    d = s.diag()
    tie = want["gap"] < NEAR_TIE
    mism = got != want["tokens"]
    assert not np.any(mism & ~tie), f"token mismatch outside near-ties: rows {np.nonzero(mism & ~tie)[0][:8]}"
    assert np.all(got[mism] == want["second"][mism])            # a near-tie may only flip to the runner-up
    assert tie.sum() <= max(1, w.R // 64)
    ok = ~mism
    assert np.abs(d["delta"] - want["delta"])[ok].max() < TOL
    assert np.abs(logW - o.logW)[ok].max() < TOL
    assert np.abs(cum - o.cumlogp)[ok].max() < TOL
    assert np.array_equal(s.live_hist()[:, t - 1], got)
    assert d["counters"][0] == 0
    res = dict(tokens=got, delta=d["delta"], counters=d["counters"], ties=int(tie.sum()))
    s.close()
    return res


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V", [1, 2, 3, 8, 9, 257, 5000, 40000])
def test_step_matches_oracle_small(dtype, V):
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=3, N=4, V=V, dtype=dtype)
    pad = (-V) % (8 if dtype == "bf16" else 4)
    for mode in (1, 0):                # every entry scored / only entries that can win
        for ww in (4, 8, 16):
            check_step(w, seed=5, t=3, alpha_t=4.0, alpha_prev=4.0, tau=-1.0, dense=mode, stride_pad=pad, wg_waves=ww)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_with_a_million_entry_vocabulary(dtype):
    """Wider than any current model: 1 048 583 entries (not a multiple of the vector width), 32 slices per row."""
    V = 1048583
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=1, N=3, V=V, dtype=dtype)
    pad = (-V) % (8 if dtype == "bf16" else 4)
    r1 = check_step(w, seed=8, t=1, alpha_t=4.0, alpha_prev=4.0, tau=-1.0, stride_pad=pad)
    r2 = check_step(w, seed=8, t=1, alpha_t=4.0, alpha_prev=4.0, tau=-1.0, stride_pad=pad, wg_waves=4, n_split=1)
    assert np.array_equal(r1["tokens"], r2["tokens"])


@pytest.mark.parametrize("name,V", [("cfg2", 152064), ("cfg3", 128256), ("cfg4", 152064), ("cfg5", 152064)])
def test_step_matches_oracle_full_vocab(name, V):
    """Full vocabulary width of every workload on a reduced number of rows; lazy and dense scoring agree."""
    base = synth.WORKLOADS[name]
    w = synth.scaled(base, B=2, N=8)
    a = base.alpha
    r1 = check_step(w, seed=1, t=2, alpha_t=a, alpha_prev=a, tau=-1.0)
    r2 = check_step(w, seed=1, t=2, alpha_t=a, alpha_prev=a, tau=-1.0, dense=1)
    assert np.array_equal(r1["tokens"], r2["tokens"])
    assert r1["counters"][1] < r2["counters"][3]        # the lazy pass scored fewer entries than it saw
    for ns, ww in ((1, 4), (3, 4), (32, 4), (1, 16), (2, 16), (7, 16), (4, 8), (9, 8)):   # launch shapes: slices per row, waves
        r3 = check_step(w, seed=1, t=2, alpha_t=a, alpha_prev=a, tau=-1.0, n_split=ns, wg_waves=ww)
        assert np.array_equal(r1["tokens"], r3["tokens"])


@pytest.mark.parametrize("alpha_t,alpha_prev,tau", [(1.0, 1.0, -1.0), (1.0234375, 1.0, -1.0), (2.5, 2.4765625, -1.0),
                                                     (4.0, 4.0, 0.5), (4.0, 3.0, 1.0), (6.0, 6.0, -1.0), (3.0, 3.0, 0.3),
                                                     (2.0, 2.0, 2.5), (10.0, 10.0, -1.0), (8.0, 8.0, -1.0), (7.0, 7.0, -1.0),
                                                     (12.0, 12.0, 0.02)])
def test_step_schedules_and_temperatures(alpha_t, alpha_prev, tau):
    """Bridging stages (non-integer exponents, boundary term) and proposals other than tau = 1/alpha."""
    for name in ("cfg4", "cfg2"):
        w = synth.scaled(synth.WORKLOADS[name], B=2, N=4, V=20000 + 8)
        for mode in (0, 1):
            check_step(w, seed=9, t=5, alpha_t=alpha_t, alpha_prev=alpha_prev, tau=tau, dense=mode)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_flat_proposals(dtype):
    """Small beta or logits that differ little: most entries may win, the candidate rings fill up and are scored while
    the row is still streaming -- same tokens as the oracle and as dense scoring."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=2, N=6, V=152064, dtype=dtype)
    x = synth.logits_numpy(synth.scaled(w, dtype="f32"), 1, 3)
    x[w.R // 2:] *= np.float32(0.125)                    # rows whose logits barely differ: flat even at beta = 4
    if dtype == "bf16":
        x = synth.f32_to_bf16_bits(x)
    for alpha, rows in ((1.0, slice(None)), (4.0, slice(w.R // 2, None))):
        for ww, ns in ((4, 1), (16, 0)):
            r1 = check_step(w, seed=3, t=1, alpha_t=alpha, alpha_prev=alpha, tau=-1.0, logits=x, wg_waves=ww, n_split=ns)
            r2 = check_step(w, seed=3, t=1, alpha_t=alpha, alpha_prev=alpha, tau=-1.0, logits=x, dense=1, wg_waves=ww, n_split=ns)
            assert np.array_equal(r1["tokens"], r2["tokens"])
            if alpha == 4.0:                             # logits within a few units of each other: nearly all must be scored
                assert r1["counters"][1] > 0.3 * r1["counters"][3]
            assert r1["counters"][2] > 0                 # the rings were drained


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_with_masked_vocabulary_entries(dtype):
    """Logit masks (-inf entries: padded vocabulary ids, constrained decoding): a masked entry has probability 0 under
    both p and q, is never drawn, and leaves the sums of the others exact -- from a third of the vocabulary masked
    to all but three entries."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=2, N=4, V=152064, dtype=dtype)
    x = synth.logits_numpy(synth.scaled(w, dtype="f32"), 1, 5)
    rng = np.random.default_rng(5)
    keep = np.ones((w.R, w.V), bool)
    keep[0:4] = rng.random((4, w.V)) > 0.33
    keep[4:6] = rng.random((2, w.V)) > 0.999
    keep[6:8] = False
    for r in (6, 7):
        keep[r, rng.choice(w.V, 3, replace=False)] = True
    keep[7, -1] = True                                        # the very last entry of a row
    x[~keep] = -np.inf
    xs = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    for alpha in (4.0, 1.5):
        for ww in (4, 16):
            res = check_step(w, seed=5, t=2, alpha_t=alpha, alpha_prev=alpha, tau=-1.0, logits=xs, wg_waves=ww)
            assert np.all(keep[np.arange(w.R), res["tokens"]])


def test_step_degenerate_rows():
    V = 4096 + 24
    w = synth.scaled(synth.WORKLOADS["cfg4"], B=1, N=6, V=V)
    x = synth.logits_numpy(w, 1, 0)
    x[0, :] = 1.5                                   # flat row: every entry can win
    x[1, :] = -80.0; x[1, 777] = 60.0               # one-hot
    x[2, :] = np.linspace(-30, 30, V)               # ascending: the running maximum rises all the way
    x[3, :] = np.linspace(30, -30, V)               # descending
    x[4, :] = 1000.0 + x[4, :]                      # large offset
    x[5, :] = -1000.0 + 1e-3 * x[5, :]              # large negative, tiny spread
    for mode, ww in ((0, 4), (0, 16), (1, 4)):
        res = check_step(w, seed=2, t=1, alpha_t=4.0, alpha_prev=4.0, tau=-1.0, logits=x, dense=mode, wg_waves=ww)
        assert res["tokens"][1] == 777


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_with_the_maximum_in_awkward_places(dtype):
    """The entry that holds the running maximum is drawn early for the bound (and scored again with its vector): rows
    whose maximum sits in the first entry, the last full vector, the ragged tail behind it, in every lane's first
    vector at once (equal maxima), or rises in steps of one batch -- same tokens and sums as the oracle, with a
    row split over slices and not."""
    V = 8 * 6000 + 3
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=1, N=8, V=V, dtype=dtype)
    x = synth.logits_numpy(synth.scaled(w, dtype="f32"), 1, 9)
    x[0, 0] = 14.0
    x[1, V - 4] = 14.0                                   # last entry of the last full vector
    x[2, V - 1] = 14.0                                   # last entry of the ragged tail
    x[3, V - 3] = 14.0                                   # first entry of the ragged tail
    x[4, 0:2048:8] = 11.0                                # every lane of the first waves starts with the same maximum
    x[5, ::4096] += 6.0                                  # a new maximum every few batches
    x[6, :] = np.float32(-3.0); x[6, V - 2] = 0.5         # flat but for one entry in the tail
    x[7, : V // 2] = -np.inf                             # the first half masked: no finite entry in the first batches
    xs = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    pad = (-V) % (8 if dtype == "bf16" else 4)
    for ww, ns in ((4, 1), (4, 3), (16, 0), (8, 2)):
        for alpha in (4.0, 1.25):
            res = check_step(w, seed=9, t=2, alpha_t=alpha, alpha_prev=alpha, tau=-1.0, logits=xs, stride_pad=pad, wg_waves=ww, n_split=ns)
            assert res["tokens"][7] >= V // 2


def test_ess_and_resample_match_oracle():
    from paper_2602_10273_amd import binding as smc
    rng = np.random.default_rng(0)
    for (B, N, kappa) in [(1, 4, 0.5), (16, 8, 0.5), (8, 16, 0.5), (64, 32, 0.5), (4, 64, 0.7), (3, 100, 0.9),
                          (2, 1024, 0.6), (5, 1, 0.5), (6, 8, 0.0), (6, 8, 1.0), (3, 33, 1.0), (1, 1, 1.0)]:
        s = Session(B, N, 64, 8, "f32", kappa, seed=123, with_hist=False)
        for scale in (0.1, 1.0, 5.0, 40.0):
            logW = rng.standard_normal(B * N) * scale
            if N >= 4:
                logW[:N] = 0.3                         # uniform prompt
            d = torch.as_tensor(logW).cuda()
            smc.smc_ess_from(s.ctx, d, s.ess, s.lognormw)
            e_ref, lnw_ref = orc.ess(logW, B, N)
            assert np.abs(s.ess.cpu().numpy() - e_ref).max() < 1e-9 * N
            assert np.abs(s.lognormw.cpu().numpy() - lnw_ref).max() < 1e-12
            for t in (1, 7):
                d2 = d.clone()
                smc.smc_resample_from(s.ctx, d2, t, s.anc, s.resampled, s.ess)
                anc_ref, flag_ref, e2, lw_ref = orc.resample(logW, B, N, kappa, 123, t)
                near = np.abs(e_ref - kappa * N) < 1e-9
                assert np.array_equal(s.resampled.cpu().numpy()[~near], flag_ref[~near])
                assert np.array_equal(s.anc.cpu().numpy(), anc_ref)          # bit-exact ancestors
                assert np.array_equal(d2.cpu().numpy(), lw_ref)
        s.close()


@pytest.mark.parametrize("scheme", ["stratified", "multinomial", "residual"])
def test_other_resampling_schemes_match_oracle(scheme):
    from paper_2602_10273_amd import binding as smc
    rng = np.random.default_rng(5)
    for (B, N) in [(6, 8), (4, 64), (3, 100), (2, 1024)]:
        s = Session(B, N, 64, 8, "f32", 1.0, seed=77, with_hist=False)      # kappa = 1: every prompt resamples
        smc.smc_set_resampler(s.ctx, orc.SCHEMES[scheme])
        for scale in (0.3, 2.0, 10.0):
            logW = rng.standard_normal(B * N) * scale
            for t in (1, 5):
                d = torch.as_tensor(logW).cuda()
                smc.smc_resample_from(s.ctx, d, t, s.anc, s.resampled, s.ess)
                anc_ref, flag_ref, _, lw_ref = orc.resample(logW, B, N, 1.0, 77, t, scheme)
                assert np.array_equal(s.resampled.cpu().numpy(), flag_ref)
                assert np.array_equal(s.anc.cpu().numpy(), anc_ref)
                assert np.array_equal(d.cpu().numpy(), lw_ref)
        s.close()


@pytest.mark.parametrize("scheme", ["systematic", "stratified", "multinomial", "residual"])
def test_survivors_in_place_order_matches_oracle(scheme):
    from paper_2602_10273_amd import binding as smc
    rng = np.random.default_rng(6)
    for (B, N) in [(5, 1), (6, 8), (4, 64), (3, 100), (2, 1024)]:
        kappa = 1.0                                                         # every prompt with N > 1 resamples
        s = Session(B, N, 64, 8, "f32", kappa, seed=78, with_hist=False)
        smc.smc_set_resampler(s.ctx, orc.SCHEMES[scheme])
        smc.smc_set_ancestor_order(s.ctx, 1)
        for scale in (0.3, 2.0, 10.0):
            logW = rng.standard_normal(B * N) * scale
            d = torch.as_tensor(logW).cuda()
            smc.smc_resample_from(s.ctx, d, 3, s.anc, s.resampled, s.ess)
            anc_ref, flag_ref, _, lw_ref = orc.resample(logW, B, N, kappa, 78, 3, scheme, in_place=True)
            anc = s.anc.cpu().numpy()
            assert np.array_equal(s.resampled.cpu().numpy(), flag_ref)
            assert np.array_equal(anc, anc_ref)
            for b in range(B):
                loc = anc[b * N:(b + 1) * N] - b * N
                assert all(loc[j] == j for j in np.unique(loc))
        with pytest.raises(Exception):
            smc.smc_set_ancestor_order(s.ctx, 2)
        s.close()


def test_resample_degenerate_weights():
    from paper_2602_10273_amd import binding as smc
    B, N = 3, 8
    s = Session(B, N, 64, 8, "f32", 0.5, seed=1, with_hist=False)
    logW = np.zeros(B * N)
    logW[0:N] = [0, -np.inf, -np.inf, -np.inf, -np.inf, -np.inf, -np.inf, -np.inf]
    logW[N:2 * N] = [-800, -900, -1000, -800, -2000, -800, -800.5, -801]
    logW[2 * N:] = 700.0
    d = torch.as_tensor(logW).cuda()
    smc.smc_resample_from(s.ctx, d, 3, s.anc, s.resampled, s.ess)
    anc_ref, flag_ref, e_ref, lw_ref = orc.resample(logW, B, N, 0.5, 1, 3)
    assert np.array_equal(s.anc.cpu().numpy(), anc_ref) and np.array_equal(s.resampled.cpu().numpy(), flag_ref)
    assert np.allclose(s.ess.cpu().numpy(), e_ref, rtol=1e-12)
    assert list(s.anc.cpu().numpy()[:N]) == [0] * N
    s.close()


@pytest.mark.parametrize("B,N,H,S,D,valid", [(3, 4, 2, 6, 16, 6), (3, 4, 2, 6, 16, 4), (4, 8, 4, 300, 128, 300),
                                              (4, 8, 4, 300, 128, 173), (2, 64, 2, 40, 64, 40), (2, 100, 1, 33, 8, 20)])
def test_reindex_bytes_exact(B, N, H, S, D, valid):
    rng = np.random.default_rng(7)
    R = B * N
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=B, N=N, H=H, S=S, D=D, layers=2)
    kv = synth.kv_numpy(w, seed=3)
    T_max = 16
    s = Session(B, N, 32, T_max, "f32", 0.5, 1, kv=kv)
    hist0 = rng.integers(0, 32, size=(R, T_max)).astype(np.int32)
    s.histA.copy_(torch.as_tensor(hist0))
    o = orc.OracleSMC(B, N, 32, T_max, 0.5, 1, "f32", kv=[k.copy() for k in kv])
    o.hist[:] = hist0
    cum = rng.standard_normal(R); o.cumlogp[:] = cum; s.set_state(None, cum)
    for it in range(3):                                     # several rounds: parity flips back and forth
        anc = np.arange(R, dtype=np.int32)
        flag = (rng.random(B) < 0.7).astype(np.int32)
        if it == 0:
            flag[0] = 1
        for b in range(B):
            if it == 1 and b == 0:
                anc[b * N:(b + 1) * N] = b * N + rng.permutation(N)                 # permutation
            else:
                anc[b * N:(b + 1) * N] = b * N + np.sort(rng.integers(0, N, N))     # duplicates
        # poison every row's inactive buffer: stale bytes must never be read as live data
        _, _, par = s.state()
        for ten in range(len(kv)):
            pa = torch.as_tensor(par.astype(bool)).cuda()
            s.kvA[ten][pa] = -21846                                         # 0xAAAA in the buffer that is not live
            s.kvB[ten][~pa] = -21846
        t = 5 + it
        # what a step does before a reindex: column t-1 of the live history receives this step's tokens
        col = rng.integers(0, 32, size=R).astype(np.int32)
        o.hist[:, t - 1] = col
        cold = torch.as_tensor(col).cuda()
        pa = torch.as_tensor(par.astype(bool)).cuda()
        s.histA[~pa, t - 1] = cold[~pa]
        s.histB[pa, t - 1] = cold[pa]
        s.reindex(valid, t, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        o.reindex(anc, flag, valid, t)
        _, cum_g, par2 = s.state()
        moved = (anc != np.arange(R)) & (np.repeat(flag, N) != 0)
        assert np.array_equal(par2, par ^ moved.astype(np.int32))      # exactly the rows that received data flip
        assert np.array_equal(cum_g, o.cumlogp)
        assert np.array_equal(s.live_hist()[:, :t], o.hist[:, :t])
        for ten in range(len(kv)):
            got = s.live_kv(ten)
            assert np.array_equal(got[:, :, :valid], o.kv[ten][:, :, :valid])
    s.close()


@pytest.mark.parametrize("eos_id,skip", [(3, 0), (-1, 0), (-1, 1)])
def test_reindex_copies_the_cache_of_terminated_ancestors_by_default(eos_id, skip):
    """Without the opt-in shortcut -- and always when no end-of-sequence token is configured, whatever flags
    smc_set_done stored -- the reorder is the plain gather: every live KV byte equals the oracle's."""
    B, N, H, S, D = 3, 6, 2, 10, 16
    R = B * N
    rng = np.random.default_rng(12)
    kv = [rng.integers(0, 65536, (R, H, S, D), dtype=np.uint16) for _ in range(2)]
    s = Session(B, N, 64, 8, "f32", 0.5, 0, kv=kv, eos_id=eos_id)
    smc.smc_set_kv_skip_terminated(s.ctx, skip)
    o = orc.OracleSMC(B, N, 64, 8, 0.5, 0, "f32", kv=[k.copy() for k in kv], eos_id=eos_id, skip_terminated_kv=bool(skip))
    for it in range(4):
        done = (rng.random(R) < 0.4).astype(np.int32)
        o.done[:] = done; s.set_done(done)
        anc = np.concatenate([b * N + np.sort(rng.integers(0, N, N)) for b in range(B)]).astype(np.int32)
        flag = np.array([1, 1, it % 2], np.int32)
        s.reindex(S, 5, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        o.reindex(anc, flag, S, 5)
        assert o.kv_specified.all()
        for ten in range(2):
            assert np.array_equal(s.live_kv(ten), o.kv[ten])
        assert np.array_equal(s.done(), o.done)
    s.close()


def test_reindex_leaves_the_cache_of_terminated_ancestors_alone():
    """smc_set_kv_skip_terminated(1).  A terminated particle is a no-op (App. D): descendants of a terminated ancestor
    get its history, sum, flag and a flipped parity like any moved row, but no KV bytes are read or written for them;
    everything else follows the oracle's gather, and the oracle (same option) names the rows it leaves unspecified."""
    B, N, H, S, D = 3, 6, 2, 10, 16
    R = B * N
    rng = np.random.default_rng(11)
    kv = [rng.integers(0, 65536, (R, H, S, D), dtype=np.uint16) for _ in range(2)]
    s = Session(B, N, 64, 8, "f32", 0.5, 0, kv=kv, eos_id=3)
    smc.smc_set_kv_skip_terminated(s.ctx, 1)
    o = orc.OracleSMC(B, N, 64, 8, 0.5, 0, "f32", kv=[k.copy() for k in kv], eos_id=3, skip_terminated_kv=True)
    o.hist[:] = rng.integers(0, 64, (R, 8)); o.cumlogp[:] = -rng.random(R)
    s.histA.copy_(torch.as_tensor(o.hist)); s.set_state(None, o.cumlogp)
    for it in range(4):
        done = (rng.random(R) < 0.4).astype(np.int32)
        o.done[:] = done; s.set_done(done)
        anc = np.concatenate([b * N + np.sort(rng.integers(0, N, N)) for b in range(B)]).astype(np.int32)
        flag = np.array([1, 1, it % 2], np.int32)
        _, _, par = s.state()
        a_before = [t.view(torch.int16).cpu().numpy().copy() for t in s.kvA]
        b_before = [t.view(torch.int16).cpu().numpy().copy() for t in s.kvB]
        o.kv = [s.live_kv(i) for i in range(2)]                  # the oracle starts from what is live on the device
        o.kv_specified[:] = True
        s.reindex(S, 5, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        o.reindex(anc, flag, S, 5)
        moved = (anc != np.arange(R)) & (np.repeat(flag, N) != 0)
        dead = ~o.kv_specified                                   # rows that continue a terminated ancestor
        assert dead.any() and (moved & ~dead).any() and not (dead & ~moved).any()
        _, cum_g, par2 = s.state()
        assert np.array_equal(par2, par ^ moved.astype(np.int32))
        assert np.array_equal(cum_g, o.cumlogp) and np.array_equal(s.done(), o.done)
        assert np.array_equal(s.live_hist()[:, :5], o.hist[:, :5])
        for ten in range(2):
            got = s.live_kv(ten)
            assert np.array_equal(got[~dead], o.kv[ten][~dead])              # every other row as the gather defines
            a_now = s.kvA[ten].view(torch.int16).cpu().numpy(); b_now = s.kvB[ten].view(torch.int16).cpu().numpy()
            assert np.array_equal(a_now[dead], a_before[ten][dead]) and np.array_equal(b_now[dead], b_before[ten][dead])
    s.close()


def test_reindex_rejects_foreign_ancestors_without_touching_memory():
    B, N = 2, 4
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=B, N=N, H=1, S=4, D=8, layers=1)
    kv = synth.kv_numpy(w, seed=3)
    s = Session(B, N, 32, 8, "f32", 0.5, 1, kv=kv)
    anc = np.array([0, 0, 7, -3, 4, 5, 6, 7], np.int32)       # rows 2,3 point outside prompt 0
    flag = np.array([1, 0], np.int32)
    s.reindex(4, 1, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
    got = s.live_kv(0)
    assert np.array_equal(got[0], kv[0][0]) and np.array_equal(got[1], kv[0][0])
    assert np.array_equal(got[2], kv[0][2]) and np.array_equal(got[3], kv[0][3])      # skipped rows keep their data
    _, _, par = s.state()
    assert list(par) == [0, 1, 0, 0, 0, 0, 0, 0]              # only row 1 received another row
    s.close()


@pytest.mark.parametrize("name,kw,eos", [("cfg2", dict(B=5, N=8, V=9000 + 8), -1), ("cfg4", dict(B=3, N=32, V=4100, ramp=6, kappa=0.999), -1),
                                         ("cfg5", dict(B=2, N=64, V=3000 + 8), -1), ("cfg2", dict(B=40, N=32, V=2048 + 8), 11),
                                         ("cfg2", dict(B=2, N=130, V=2048), -1)])
def test_step_resample_in_one_launch_equals_the_two_calls(name, kw, eos):
    """smc_step_resample (the row finalizer's wave goes on to resample its prompt) against smc_step + smc_resample on a
    second context: same tokens, ancestors, flags, ESS, weights, sums and estimate of log Z after every step, for every
    resampling scheme and both ancestor orders."""
    w = synth.scaled(synth.WORKLOADS[name], **kw)
    for scheme, order in ((0, 0), (1, 0), (2, 1), (3, 0), (0, 1)):
        a = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, 21, with_hist=True, eos_id=eos)
        b = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, 21, with_hist=True, eos_id=eos)
        for s in (a, b):
            smc.smc_set_resampler(s.ctx, scheme); smc.smc_set_ancestor_order(s.ctx, order)
        n_res = 0
        for t in range(1, 7):
            x = to_device_logits(synth.logits_numpy(w, t, 21), w.dtype)
            a.step(x, t, w.alpha_at(t), w.alpha_at(t - 1)); a.resample(t)
            b.step_resample(x, t, w.alpha_at(t), w.alpha_at(t - 1))
            for s in (a, b):
                s.reindex(0, t)
            torch.cuda.synchronize()
            for f in ("tokens", "anc", "resampled", "ess"):
                assert torch.equal(getattr(a, f), getattr(b, f)), (scheme, order, t, f)
            sa, sb = a.state(), b.state()
            assert np.array_equal(sa[0], sb[0]) and np.array_equal(sa[1], sb[1])
            assert np.array_equal(a.log_Zhat(), b.log_Zhat())
            if eos >= 0:
                assert np.array_equal(a.done(), b.done())
            n_res += int(a.resampled.sum())
        assert n_res > 0
        assert np.array_equal(a.live_hist(), b.live_hist())
        a.close(); b.close()


@pytest.mark.parametrize("B,N,V,eos,order", [(64, 16, 2048 + 8, -1, 0), (40, 32, 1024 + 8, 7, 0), (5, 8, 4096 + 8, -1, 1),
                                             (33, 32, 1024, -1, 1), (3, 400, 1024 + 8, 5, 0)])
def test_step_resample_reindex_equals_the_separate_calls(B, N, V, eos, order):
    """smc_step_resample_reindex (three launches at every size: from 1024 rows on the wave that resamples a prompt goes
    on to plan its reorder) against smc_step_resample + smc_kv_reindex on a second context: tokens, ancestors, flags,
    ESS, weights, sums, parities, termination flags, histories and every KV byte after every step, with a partly
    filled cache and with the survivors-in-place ancestor order."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=B, N=N, V=V, H=2, S=12, D=16, layers=1, kappa=0.9)
    kv = synth.kv_numpy(w, 3)
    a = Session(w.B, w.N, w.V, 12, w.dtype, w.kappa, 3, kv=[k.copy() for k in kv], eos_id=eos)
    b = Session(w.B, w.N, w.V, 12, w.dtype, w.kappa, 3, kv=[k.copy() for k in kv], eos_id=eos)
    for s in (a, b):
        smc.smc_set_ancestor_order(s.ctx, order)
    n_res = 0
    for t in range(1, 9):
        x = to_device_logits(synth.logits_numpy(w, t, 3), w.dtype)
        valid = min(t + 3, w.S)
        a.step_resample(x, t, w.alpha, w.alpha); a.reindex(valid, t)
        b.step_resample_reindex(x, t, w.alpha, w.alpha, valid)
        torch.cuda.synchronize()
        for f in ("tokens", "anc", "resampled", "ess"):
            assert torch.equal(getattr(a, f), getattr(b, f)), (t, f)
        sa, sb = a.state(), b.state()
        for u, v in zip(sa, sb):
            assert np.array_equal(u, v), t
        if eos >= 0:
            assert np.array_equal(a.done(), b.done())
        n_res += int(a.resampled.sum())
    assert n_res > 0
    assert np.array_equal(a.live_hist(), b.live_hist())
    for ten in range(len(kv)):
        assert np.array_equal(a.live_kv(ten), b.live_kv(ten))
    a.close(); b.close()


def test_tickets_hand_every_record_over_on_many_contended_steps():
    """Rows split over many slices and prompts of many rows, thousands of workgroups, 150 free-running steps.  Three runs
    on the same logits: (a) eight slices per row, resampling in a launch of its own; (b) eight slices per row, slices
    and prompts joined through tickets inside one launch (agent-scope stores of the records and the weights, then the
    ticket); (c) every row in one slice, no ticket anywhere.  (a) and (b) merge the same records in the same order, so
    they must agree to the last bit in everything; (c) sums in another order, so its draws are compared where no
    near-tie decides them and its sums to rounding.  A record or a weight read before it was written would show as a
    wrong sum, weight or ancestor."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=8, N=64, V=8192 + 8, kappa=0.9)
    a, b, c = (Session(w.B, w.N, w.V, 160, w.dtype, w.kappa, 5, with_hist=False) for _ in range(3))
    smc.smc_set_tuning(a.ctx, 8, 0, 4)
    smc.smc_set_tuning(b.ctx, 8, 0, 4)
    smc.smc_set_tuning(c.ctx, 1, 0, 4)
    xs = [to_device_logits(synth.logits_numpy(w, t, 5), w.dtype) for t in range(1, 9)]
    n_res = 0
    for t in range(1, 151):
        x = xs[t % 8]
        a.step(x, t, w.alpha, w.alpha); a.resample(t)
        b.step_resample(x, t, w.alpha, w.alpha)
        c.step(x, t, w.alpha, w.alpha)
        torch.cuda.synchronize()
        for f in ("tokens", "anc", "resampled", "ess"):
            assert torch.equal(getattr(a, f), getattr(b, f)), (t, f)
        sa, sb, sc = a.state(), b.state(), c.state()
        assert np.array_equal(sa[0], sb[0]) and np.array_equal(sa[1], sb[1]), t
        ga, gc = a.diag()["gap"], c.diag()["gap"]
        clear = (ga > 1e-4) & (gc > 1e-4)
        assert clear.mean() > 0.99
        assert np.array_equal(a.tokens.cpu().numpy()[clear], c.tokens.cpu().numpy()[clear]), t
        if clear.all():                                   # (c has not resampled: compare the weights a had before it did)
            da = a.diag()
            np.testing.assert_allclose(da["delta"], c.diag()["delta"], rtol=0, atol=1e-5)
            np.testing.assert_allclose(sa[1], sc[1], rtol=0, atol=1e-5)
        c.set_state(sa[0], sa[1])                         # in step again, so that rounding cannot build up
        n_res += int(a.resampled.sum())
    assert n_res > 20
    a.close(); b.close(); c.close()
