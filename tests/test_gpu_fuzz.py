"""Seeded random sweep of the vocabulary pass and of the reorder: shapes, row strides, exponents, proposal
temperatures, launch shapes and logit distributions drawn at random, each case compared with the oracle to the same
bars as the component tests (tokens bit-exact outside oracle-flagged near-ties, weights within 1e-4, bytes exact)."""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2602_10273_amd import binding as smc
from paper_2602_10273_amd import synth
from paper_2602_10273_amd.harness import Session, to_device_logits

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _random_logits(rng, R, V, dtype):
    kind = rng.integers(0, 8)
    scale = float(rng.uniform(0.3, 6.0))
    if kind == 0:
        x = rng.standard_normal((R, V)) * scale
    elif kind == 1:
        x = rng.standard_t(3, (R, V)) * scale
    elif kind == 2:                                           # a few dominant tokens
        x = rng.standard_normal((R, V)) * 0.5
        for r in range(R):
            x[r, rng.integers(0, V, size=min(V, 3))] += rng.uniform(5, 30)
    elif kind == 3:                                           # sorted rows: the running maximum keeps rising / never rises
        x = np.sort(rng.standard_normal((R, V)) * scale, axis=1)
        if rng.random() < 0.5:
            x = x[:, ::-1]
    elif kind == 4:                                           # masked-out tokens and a large common offset
        x = rng.standard_normal((R, V)) * scale + rng.uniform(-500, 500)
        x[rng.random((R, V)) < 0.3] = -np.inf
        x[:, rng.integers(0, V)] = rng.uniform(-2, 2)         # at least one finite entry per row
    elif kind == 5:                                           # heavy ties: few distinct values
        x = rng.integers(-3, 4, (R, V)).astype(np.float64) * scale
    elif kind == 6:                                           # all but a handful of entries masked: whole slices are empty
        x = np.full((R, V), -np.inf)
        for r in range(R):
            idx = rng.choice(V, size=min(V, int(rng.integers(1, 6))), replace=False)
            x[r, idx] = rng.standard_normal(idx.size) * scale
    else:                                                     # logits that barely differ: every entry can win
        x = rng.standard_normal((R, V)) * rng.uniform(0.01, 0.2) + rng.uniform(-50, 50)
    x = np.ascontiguousarray(x, np.float32)
    return synth.f32_to_bf16_bits(x) if dtype == "bf16" else x


@pytest.mark.parametrize("case", range(72))
def test_vocab_pass_random_case(case):
    rng = np.random.default_rng([2602, case])
    dtype = "bf16" if rng.random() < 0.5 else "f32"
    epv = 8 if dtype == "bf16" else 4
    B = int(rng.integers(1, 5)); N = int(rng.integers(1, 9))
    V = int(rng.choice([1, 2, 7, 63, 64, 65, 255, 1023, 1025, 4096, 4097, int(rng.integers(2, 30000)), int(rng.integers(30000, 70000))]))
    R = B * N
    pad = (-V) % epv + epv * int(rng.integers(0, 4))
    x = _random_logits(rng, R, V, dtype)
    xs = np.concatenate([x, np.full((R, pad), 0x7FC0 if dtype == "bf16" else np.nan, x.dtype)], axis=1) if pad else x
    alpha_t = float(rng.choice([1.0, 2.0, 4.0, 6.0, 1.0 + 3.0 * rng.random()]))
    alpha_prev = alpha_t if rng.random() < 0.6 else max(1.0, alpha_t - rng.random())
    tau = -1.0 if rng.random() < 0.6 else float(rng.uniform(0.15, 1.5))
    n_split = int(rng.choice([0, 1, 2, 3, 5, 32])); ww = int(rng.choice([0, 4, 16])); dense = int(rng.random() < 0.25)
    t = int(rng.integers(1, 8)); seed = int(rng.integers(0, 2 ** 40))
    eos = int(rng.integers(0, V)) if rng.random() < 0.3 else -1
    print(dict(case=case, dtype=dtype, B=B, N=N, V=V, pad=pad, alpha_t=alpha_t, alpha_prev=alpha_prev, tau=tau,
               n_split=n_split, wg_waves=ww, dense=dense, t=t, seed=seed, eos=eos), flush=True)
    o = orc.OracleSMC(B, N, V, 8, 0.5, seed, dtype, eos_id=eos)
    o.logW[:] = rng.standard_normal(R); o.cumlogp[:] = -rng.random(R) * 5
    if eos >= 0:
        o.done[:] = (rng.random(R) < 0.3).astype(np.int32)
    s = Session(B, N, V, 8, dtype, 0.5, seed, eos_id=eos)
    s.set_state(o.logW, o.cumlogp)
    if eos >= 0:
        s.set_done(o.done)
    smc.smc_set_tuning(s.ctx, n_split, dense, ww)
    want = o.step(xs, t, alpha_t, alpha_prev, tau, row_stride=xs.shape[1])
    s.step(to_device_logits(xs, dtype), t, alpha_t, alpha_prev, tau)
    got = s.tokens.cpu().numpy()
    logW, cum, _ = s.state()
    tie = want["gap"] < 1e-6
    mism = got != want["tokens"]
    assert not np.any(mism & ~tie), np.nonzero(mism & ~tie)[0][:8]
    assert np.all(got[mism] == want["second"][mism])
    ok = ~mism
    assert np.abs(logW - o.logW)[ok].max(initial=0.0) < TOL and np.abs(cum - o.cumlogp)[ok].max(initial=0.0) < TOL
    assert np.array_equal(s.live_hist()[:, t - 1], got)
    if eos >= 0:
        assert np.array_equal(s.done()[ok], o.done[ok])
    assert s.diag()["counters"][0] == 0
    s.close()


@pytest.mark.parametrize("case", range(16))
def test_reorder_random_case(case):
    rng = np.random.default_rng([10273, case])
    B = int(rng.integers(1, 6)); N = int(rng.choice([1, 2, 3, 8, 17, 64, 65, 130]))
    H = int(rng.integers(1, 4)); S = int(rng.integers(1, 40)); D = int(rng.choice([8, 16, 24, 64])); n_t = int(rng.integers(1, 4))
    R = B * N
    T_max = 16
    print(dict(case=case, B=B, N=N, H=H, S=S, D=D, n_t=n_t), flush=True)
    kv = [rng.integers(0, 65536, (R, H, S, D), dtype=np.uint16) for _ in range(n_t)]
    s = Session(B, N, 64, T_max, "f32", 0.5, 0, kv=kv)
    o = orc.OracleSMC(B, N, 64, T_max, 0.5, 0, "f32", kv=[k.copy() for k in kv])
    o.hist[:] = rng.integers(0, 64, (R, T_max)); o.cumlogp[:] = -rng.random(R)
    s.histA.copy_(torch.as_tensor(o.hist)); s.set_state(None, o.cumlogp)
    for rnd in range(5):
        flag = (rng.random(B) < 0.7).astype(np.int32)
        style = rng.integers(0, 3)
        anc = np.concatenate([b * N + (np.sort(rng.integers(0, N, N)) if style == 0 else rng.integers(0, N, N) if style == 1
                                       else rng.permutation(N)) for b in range(B)]).astype(np.int32)
        valid = int(rng.integers(0, S + 1)); t = int(rng.integers(0, T_max + 1))
        before = [s.live_kv(i) for i in range(n_t)]
        hist_before = s.live_hist()
        o.kv = [b.copy() for b in before]; o.hist = hist_before.copy()      # beyond valid / t the copy is unspecified
        o.reindex(anc, flag, valid, t)
        s.reindex(valid, t, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        moved = (anc != np.arange(R)) & (np.repeat(flag, N) != 0)
        for i in range(n_t):
            live = s.live_kv(i)
            assert np.array_equal(live[:, :, :valid], o.kv[i][:, :, :valid]), (rnd, i)
            assert np.array_equal(live[~moved], before[i][~moved])          # rows that did not move are untouched
        assert np.array_equal(s.live_hist()[:, :t], o.hist[:, :t])
        _, cum, _ = s.state()
        assert np.array_equal(cum, o.cumlogp)
    s.close()
