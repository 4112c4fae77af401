"""End-to-end and robustness checks of the HIP path that do not lean on the oracle's implementation:
the brute-force power target on the tiny bigram model, non-finite logits, two contexts on two streams."""
import numpy as np
import pytest
import torch

from oracle.enumerate import enumerate_power_target
from paper_2602_10273_amd import binding as smc
from paper_2602_10273_amd import synth
from paper_2602_10273_amd.harness import Session, to_device_logits

pytestmark = pytest.mark.gpu
W1 = synth.WORKLOADS["cfg1"]
TABLE = synth.bigram_table(W1.V, W1.sigma, seed=0)


def _run_bigram_gpu(B, N, T, alphas, seed, eos_id=-1, scheme=0):
    """Alg. 1 on the device for B independent copies of the prompt; returns (session, log Zhat per prompt)."""
    w = synth.scaled(W1, B=B, N=N)
    s = Session(B, N, w.V, 8, "f32", 0.5, seed, eos_id=eos_id)
    smc.smc_set_resampler(s.ctx, scheme)
    table_d = torch.as_tensor(TABLE).cuda()
    prev = torch.zeros(w.R, dtype=torch.long, device="cuda")
    for t in range(1, T + 1):
        x = table_d[prev].contiguous()
        s.step(x, t, alphas[t], alphas[t - 1])
        s.resample(t)                 # banks the mean unnormalised weight of every prompt that resamples
        s.reindex(0, t)
        hist = torch.as_tensor(s.live_hist()[:, t - 1]).cuda()
        prev = hist.long()
    return s, s.log_Zhat()            # the library's own estimate: banked factors times the current mean weight


@pytest.mark.parametrize("mode", ["constant", "ramp", "eos", "residual"])
def test_device_estimate_of_the_normalising_constant_is_unbiased(mode):
    """E[Zhat] = Z_alpha = sum_y p(y)^alpha, with Z_alpha from explicit enumeration of all 8^6 sequences."""
    T, a = W1.steps, W1.alpha
    eos = 3 if mode == "eos" else -1
    alphas = [1.0, 2.0, 3.0, 4.0, 4.0, 4.0, 4.0] if mode == "ramp" else [a] * (T + 1)
    _, _, log_Z = enumerate_power_target(TABLE, T, a, eos_id=eos)
    B = 20000
    s, lz = _run_bigram_gpu(B, W1.N, T, alphas, seed=97, eos_id=eos, scheme=3 if mode == "residual" else 0)
    z = np.exp(lz - log_Z)
    se = z.std(ddof=1) / np.sqrt(B)
    assert abs(z.mean() - 1.0) < 4 * se and se < 0.05, (z.mean(), se)
    s.close()


def test_device_output_draw_follows_the_power_target():
    T, a = W1.steps, W1.alpha
    seqs, log_pi, _ = enumerate_power_target(TABLE, T, a)
    B, N = 3000, 128
    s, _ = _run_bigram_gpu(B, N, T, [a] * (T + 1), seed=5)
    s.final_draw(T)
    pick = s.choice.cpu().numpy()
    chosen = s.live_hist()[pick, :T]
    for k in np.argsort(-log_pi)[:4]:
        p = np.exp(log_pi[k])
        freq = np.mean(np.all(chosen == seqs[k][None, :], axis=1))
        assert abs(freq - p) < 4 * np.sqrt(p * (1 - p) / B) + 0.03 * p
    s.close()


def test_non_finite_logits_are_flagged_and_contained():
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=2, N=4, V=4096)
    x = synth.bf16_bits_to_f32(synth.logits_numpy(w, 1, 0)).copy()
    x[1, 100] = np.nan
    x[2, 7] = np.inf
    x[5, :] = -np.inf
    x[6, 50:60] = -np.inf                     # masked-out tokens are fine
    s = Session(w.B, w.N, w.V, 8, "f32", 0.5, 3)
    s.step(to_device_logits(x, "f32"), 1, 4.0, 4.0)
    d = s.diag()
    tok = s.tokens.cpu().numpy()
    assert d["counters"][0] == 3              # rows 1, 2, 5
    assert tok[1] == 0 and tok[2] == 0 and tok[5] == 0
    good = [0, 3, 4, 6, 7]
    assert np.all(np.isfinite(d["delta"][good])) and np.all(tok[good] >= 0) and np.all(tok[good] < w.V)
    assert not (50 <= tok[6] < 60)
    s.resample(1)                             # NaN weights never trigger resampling of their prompt
    flag = s.resampled.cpu().numpy()
    assert flag[0] == 0
    s.close()


def test_two_contexts_on_two_streams_do_not_interfere():
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=4, N=8, V=30000, layers=1, H=2, S=16, D=64)
    xs = [to_device_logits(synth.logits_numpy(w, t, 0), w.dtype) for t in range(1, 5)]
    kv = synth.kv_numpy(w, 1)

    def run(stream, seed):
        with torch.cuda.stream(stream):
            s = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, seed, kv=kv, stream=stream)
            for t in range(1, 5):
                s.step(xs[t - 1], t, w.alpha, w.alpha)
                s.resample(t)
                s.reindex(w.S, t)
        return s

    torch.cuda.synchronize()
    st1, st2 = torch.cuda.Stream(), torch.cuda.Stream()
    a1, a2 = run(st1, 11), run(st2, 22)       # enqueued back to back on different streams
    torch.cuda.synchronize()
    b1 = run(torch.cuda.current_stream(), 11)
    b2 = run(torch.cuda.current_stream(), 22)
    torch.cuda.synchronize()
    for a, b in ((a1, b1), (a2, b2)):
        assert np.array_equal(a.tokens.cpu().numpy(), b.tokens.cpu().numpy())
        assert np.array_equal(a.state()[0], b.state()[0]) and np.array_equal(a.state()[2], b.state()[2])
        assert np.array_equal(a.live_hist(), b.live_hist())
        assert np.array_equal(a.live_kv(0), b.live_kv(0))
    for s in (a1, a2, b1, b2):
        s.close()


def test_hbm_probe_reports_plausible_ceilings():
    """The measurement helper: four read:write mixes over a 1 GiB buffer, all of the order of an MI355X's HBM rate
    (wide bounds: a quarter of the buffer fits the last-level cache, and the box may be busy)."""
    from paper_2602_10273_amd import binding as smc
    n = 1 << 30
    buf = torch.empty(n, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    rates = [smc.smc_hbm_probe(kind, buf, n, stream) for kind in range(4)]
    assert all(500.0 < r < 12000.0 for r in rates), rates
    assert rates[0] > rates[1]                                  # reads stream faster than writes on this device
    for bad in (lambda: smc.smc_hbm_probe(4, buf, n, stream), lambda: smc.smc_hbm_probe(0, buf, 1000, stream),
                lambda: smc.smc_hbm_probe(0, buf.data_ptr() + 8, n - 64, stream)):
        with pytest.raises(smc.SMCError):
            bad()


def test_checkpoint_and_resume_reproduce_the_uninterrupted_run():
    """The state of a run is small and explicit (weights, cumulative log p, termination flags, live histories and
    caches) and the random stream is keyed by (seed, step, row): a run restored from a snapshot into a fresh context
    continues exactly like the uninterrupted one."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=6, N=8, V=4104, layers=1, H=2, S=24, D=64)
    T, cut, seed = 20, 9, 13
    kv = synth.kv_numpy(w, 4)

    def advance(s, t0, t1):
        for t in range(t0, t1 + 1):
            s.step(to_device_logits(synth.logits_numpy(w, t, seed), w.dtype), t, w.alpha, w.alpha)
            s.resample(t)
            s.reindex(w.S, t)

    def snapshot(s, t):
        logW, cum, _ = s.state()
        return dict(logW=logW, cum=cum, done=s.done(), hist=s.live_hist(), kv=[s.live_kv(i) for i in range(len(kv))],
                    tokens=s.tokens.cpu().numpy(), banked=s.banked_log_Zhat(), logZ=s.log_Zhat())

    full = Session(w.B, w.N, w.V, T, w.dtype, w.kappa, seed, kv=kv, eos_id=7)
    advance(full, 1, cut)
    snap = snapshot(full, cut)
    advance(full, cut + 1, T)
    want = snapshot(full, T)
    full.close()

    resumed = Session(w.B, w.N, w.V, T, w.dtype, w.kappa, seed, kv=snap["kv"], eos_id=7)   # live rows go to buffer A
    resumed.histA.copy_(torch.as_tensor(snap["hist"]))
    resumed.set_state(snap["logW"], snap["cum"])
    resumed.set_done(snap["done"])
    resumed.set_banked_log_Zhat(snap["banked"])
    advance(resumed, cut + 1, T)
    got = snapshot(resumed, T)
    resumed.close()
    assert np.array_equal(got["tokens"], want["tokens"]) and np.array_equal(got["hist"][:, :T], want["hist"][:, :T])
    assert np.array_equal(got["logW"], want["logW"]) and np.array_equal(got["cum"], want["cum"])
    assert np.array_equal(got["done"], want["done"])
    assert 0 < (want["done"] == 0).sum() < w.R
    for a, b in zip(got["kv"], want["kv"]):
        assert np.array_equal(a, b)                                # every row, terminated or not (no shortcut is on)
    assert np.array_equal(got["banked"], want["banked"]) and np.array_equal(got["logZ"], want["logZ"])
    assert np.abs(want["banked"]).max() > 0
