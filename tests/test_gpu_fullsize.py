"""Parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times (automatic
launch shape, device-generated inputs downloaded for the oracle).

Vocabulary pass + weights + resampling: every row of cfg2/cfg3/cfg5, a sample of rows of cfg4 (2048 rows), one step
each with the workload's exponent, compared element by element with the oracle on the same logits.
KV reindex: the full cfg2 cache (2 x 15 GB), and the full row geometry of cfg3/cfg4/cfg5 on a reduced number of
layers (memory), checked on sampled destination rows against the source rows the ancestors name, plus properties that
hold at any size (prompts that did not resample are untouched, parity flips exactly for resampled prompts).
"""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2602_10273_amd import binding as smc
from paper_2602_10273_amd import synth
from paper_2602_10273_amd.harness import Session

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _to_numpy_logits(x, dtype):
    if dtype == "bf16":
        return x.view(torch.int16).cpu().numpy().view(np.uint16)
    return x.cpu().numpy()


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg5", "cfg4"])
def test_full_size_step_weights_and_resampling(name):
    w = synth.WORKLOADS[name]
    seed, t = 7, 3
    a_t = w.alpha if name != "cfg4" else w.alpha_at(96)          # a stage in the middle of the ramp: beta = 3.25
    a_p = a_t if name != "cfg4" else w.alpha_at(95)
    s = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, seed)
    x = synth.logits_torch(w, 1, seed)
    rng = np.random.default_rng(1)
    logW0 = rng.standard_normal(w.R) * 0.5
    cum0 = -rng.random(w.R) * 20
    s.set_state(logW0, cum0)
    s.step(x, t, a_t, a_p, -1.0)
    s.resample(t)
    tokens = s.tokens.cpu().numpy()
    d = s.diag()
    anc = s.anc.cpu().numpy(); flag = s.resampled.cpu().numpy(); ess = s.ess.cpu().numpy()
    logW_after, cum_after, _ = s.state()
    assert d["counters"][0] == 0

    rows = np.arange(w.R) if w.R <= 256 else np.sort(rng.choice(w.R, 160, replace=False))
    xh = _to_numpy_logits(x[torch.as_tensor(rows).cuda()], w.dtype)
    beta = orc.beta_of(a_t, -1.0)
    n_tie = 0
    want_logW = np.full(w.R, np.nan)
    for k, r in enumerate(rows):
        o = orc.vocab_row(xh[k], w.dtype, beta, a_t, seed, t, int(r))
        if tokens[r] != o["token"]:
            assert o["gap"] < 1e-6 and tokens[r] == o["second"], (r, tokens[r], o)
            n_tie += 1
        assert abs(d["delta"][r] - o["delta"]) < TOL
        assert abs(d["logZ1"][r] - o["logZ1"]) < TOL and abs(d["logZb"][r] - o["logZb"]) < TOL
        want_logW[r] = logW0[r] + (a_t - a_p) * cum0[r] + o["delta"]
        assert abs(cum_after[r] - (cum0[r] + o["logp"])) < TOL
    assert n_tie <= 1
    # ESS / trigger / ancestors for prompts whose rows were all checked, from the oracle's own weights
    done = [b for b in range(w.B) if np.all(np.isfinite(want_logW[b * w.N:(b + 1) * w.N]))]
    assert len(done) >= min(w.B, 2) or w.R > 256
    for b in done:
        sl = slice(b * w.N, (b + 1) * w.N)
        e_only, lnw = orc.ess(want_logW[sl], 1, w.N)
        assert abs(ess[b] - e_only[0]) < TOL
        if abs(e_only[0] - w.kappa * w.N) > TOL:
            fire = e_only[0] < w.kappa * w.N
            assert flag[b] == int(fire)
            if fire:
                u0 = orc.uniform(orc.random_word(seed, t, b, 0, 1))
                wn = np.exp(lnw)
                A = orc.systematic(wn, u0)
                C = np.cumsum(wn); p = (u0 + np.arange(w.N)) / w.N
                if np.abs(C[None, :] - p[:, None]).min() > 1e-5:        # positions not within rounding of a boundary
                    assert np.array_equal(anc[sl], b * w.N + A)
                assert np.all(logW_after[sl] == 0.0)
            else:
                assert np.array_equal(anc[sl], np.arange(b * w.N, (b + 1) * w.N))
                assert np.abs(logW_after[sl] - want_logW[sl]).max() < TOL
    s.close()


@pytest.mark.parametrize("name,layers", [("cfg2", 28), ("cfg3", 2), ("cfg4", 2), ("cfg5", 2)])
def test_full_size_reindex_sampled_rows(name, layers):
    base = synth.WORKLOADS[name]
    w = synth.scaled(base, layers=layers)
    rng = np.random.default_rng(3)
    s = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, 0, kv_geom=(w.kv_tensors, w.H, w.S, w.D), with_hist=True)
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    for ten in s.kvA:
        ten.view(torch.int16).random_(-32768, 32767, generator=g)
    for ten in s.kvB:
        ten.view(torch.int16).fill_(-21846)                      # poison 0xAAAA
    # ancestors like ESS-triggered systematic resampling produces: sorted, with duplicates; a few prompts untouched
    anc = np.arange(w.R, dtype=np.int32)
    flag = (rng.random(w.B) < 0.8).astype(np.int32); flag[0] = 1
    if w.B > 1:
        flag[1] = 0
    for b in range(w.B):
        anc[b * w.N:(b + 1) * w.N] = b * w.N + np.sort(rng.choice(w.N, size=w.N, p=rng.dirichlet(np.full(w.N, 0.5))))
    t = 5
    s.reindex(w.S, t, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
    _, _, par = s.state()
    moved = (anc != np.arange(w.R)) & (np.repeat(flag, w.N) != 0)
    assert np.array_equal(par, moved.astype(np.int32))           # rows that are their own ancestor do not move
    check_rows = np.concatenate([rng.choice(np.nonzero(moved)[0], 8, replace=False), np.nonzero(~moved)[0][:3]])
    for ten in rng.choice(w.kv_tensors, size=min(3, w.kv_tensors), replace=False):
        for r in check_rows:
            r = int(r)
            if moved[r]:
                assert torch.equal(s.kvB[ten][r].view(torch.int16), s.kvA[ten][int(anc[r])].view(torch.int16)), (ten, r)
            else:
                assert bool((s.kvB[ten][r].view(torch.int16) == -21846).all())     # untouched
    # whole-tensor property on one tensor: every moved row equals its ancestor's row
    ten = 0
    idx = torch.as_tensor(anc.astype(np.int64)).cuda()
    sel = torch.as_tensor(moved).cuda()
    want = s.kvA[ten].view(torch.int16).index_select(0, idx)      # bit patterns (random bits include NaNs)
    assert torch.equal(s.kvB[ten].view(torch.int16)[sel], want[sel])
    del want
    s.close()


@pytest.mark.parametrize("name,P", [("cfg2", 16), ("cfg5", 16), ("cfg4", 64), ("cfg3", 128)])
def test_full_size_paged_reorder(name, P):
    """Paged cache at the full row geometry (one layer): tables, counts and slots against the CPU model at every step,
    the logical content of the whole cache against a dense copy kept with index_select."""
    from oracle.paged import PagedKV
    w = synth.scaled(synth.WORKLOADS[name], layers=1)
    steps = 24
    len0 = w.S - steps - 3
    rng = np.random.default_rng(8)
    s = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, 0, kv_geom=(2, w.H, w.S, w.D), with_hist=False, page_len=P, len0=len0)
    pk = PagedKV(w.B, w.N, w.H, w.S, w.D, P, 0)                 # tables only: the content is checked against `dense`
    pk.reset(len0)
    g = torch.Generator(device="cuda"); g.manual_seed(12)
    for pool in s.pools:
        pool.view(torch.int16).random_(-32768, 32767, generator=g)

    def logical(ten, table, length):
        ncol = (length + P - 1) // P
        idx = torch.as_tensor(table[:, :ncol].astype(np.int64)).cuda()
        pages = s.pools[ten].view(torch.int16)[idx]             # [R, ncol, H, P, D]
        return pages.permute(0, 2, 1, 3, 4).reshape(w.R, w.H, ncol * P, w.D)[:, :, :length]

    table, refcnt = s.paged_state()
    assert np.array_equal(table, pk.table) and np.array_equal(refcnt, pk.refcnt)
    dense = [logical(ten, table, len0).clone() for ten in range(2)]
    dense = [torch.cat([d, torch.zeros((w.R, w.H, w.S - len0, w.D), dtype=torch.int16, device="cuda")], dim=2) for d in dense]
    copied = 0
    for i in range(steps):
        pos = len0 + i
        slot_ref, copies = pk.prepare_append(pos)
        copied += len(copies)
        s.prepare_append(pos)
        assert np.array_equal(s.slot.cpu().numpy(), slot_ref), pos
        for ten in range(2):
            new = torch.randint(-32768, 32767, (w.R, w.H, w.D), dtype=torch.int16, device="cuda", generator=g)
            s.pools[ten].view(torch.int16)[s.slot.long(), :, pos % P, :] = new
            dense[ten][:, :, pos, :] = new
        flag = (rng.random(w.B) < 0.7).astype(np.int32)
        anc = np.arange(w.R, dtype=np.int32)
        for b in range(w.B):
            if flag[b]:
                anc[b * w.N:(b + 1) * w.N] = b * w.N + np.sort(rng.choice(w.N, size=w.N, p=rng.dirichlet(np.full(w.N, 0.5))))
        pk.reindex(anc, flag)
        s.paged_reindex(0, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        idx = torch.as_tensor(anc.astype(np.int64)).cuda()
        dense = [d.index_select(0, idx) for d in dense]
        table, refcnt = s.paged_state()
        ncol = (pos + 1 + P - 1) // P
        assert np.array_equal(table[:, :ncol], pk.table[:, :ncol]) and np.array_equal(refcnt, pk.refcnt), pos
    assert copied > 0 and smc.smc_paged_check(s.ctx) == 0
    for ten in range(2):
        assert torch.equal(logical(ten, table, len0 + steps), dense[ten][:, :, :len0 + steps]), ten
    s.close()


@pytest.mark.parametrize("name,paged", [("cfg2", 0), ("cfg2", 16), ("cfg5", 0), ("cfg4", 64), ("cfg3", 0)])
def test_full_size_attention_sampled_rows(name, paged):
    """Decode attention at the full row geometry of a workload (one layer), sampled rows against the fp64 oracle."""
    from oracle.attention import decode_attention
    w = synth.scaled(synth.WORKLOADS[name], layers=1)
    G = 7 if w.H == 4 else 4
    Hq = G * w.H
    s = Session(w.B, w.N, w.V, 8, w.dtype, w.kappa, 0, kv_geom=(2, w.H, w.S, w.D), with_hist=False, page_len=paged, len0=w.S)
    g = torch.Generator(device="cuda"); g.manual_seed(21)
    for t in (s.pools if paged else s.kvA):
        t.normal_(generator=g)
    rng = np.random.default_rng(4)
    if not paged:                                                # rows in both buffers
        flag = torch.ones(w.B, dtype=torch.int32, device="cuda")
        s.reindex(w.S, 0, torch.as_tensor(synth.ancestors_numpy(w, 1)).cuda(), flag)
    q = torch.randn((w.R, Hq, w.D), device="cuda", generator=g).to(torch.bfloat16)
    scale = float(w.D) ** -0.5
    for length in (w.S, w.S - 37):
        out = s.attention(0, 1, q, length, scale).cpu().numpy()
        rows = rng.choice(w.R, size=3, replace=False)
        if paged:
            table, _ = s.paged_state()
            ncol = (w.S + paged - 1) // paged
            def dense(ten, r):
                pg = s.pools[ten].view(torch.int16)[torch.as_tensor(table[r, :ncol].astype(np.int64)).cuda()]   # [ncol, H, P, D]
                return pg.permute(1, 0, 2, 3).reshape(w.H, ncol * paged, w.D)[:, :w.S].cpu().numpy().view(np.uint16)
            kb = np.stack([dense(0, int(r)) for r in rows]); vb = np.stack([dense(1, int(r)) for r in rows])
        else:
            kb = s.live_kv(0, rows); vb = s.live_kv(1, rows)
        qb = q[torch.as_tensor(rows).cuda()].view(torch.int16).cpu().numpy().view(np.uint16)
        want = decode_attention(qb, kb, vb, length, scale)
        assert np.abs(out[rows] - want).max() < TOL, (length, np.abs(out[rows] - want).max())
    s.close()
