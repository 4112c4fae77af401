"""Paged form of the cache reorder: HIP path vs the CPU model that follows the same allocation rules, and vs the
dense row gather that defines the reorder (Alg. 1 "reorder KV cache by A"; App. C).  Tables, reference counts and
slots bit-exact; logical cache content bit-exact."""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from oracle.paged import PagedKV
from paper_2602_10273_amd import binding as smc
from paper_2602_10273_amd import synth
from paper_2602_10273_amd.harness import Session, to_device_logits

pytestmark = pytest.mark.gpu


def _logical(s, ten, table, length):
    """[R, H, length, D] uint16 read through the table from the device pools."""
    P = s.page_len
    ncol = (length + P - 1) // P
    pool = s.pools[ten].view(torch.int16)
    idx = torch.as_tensor(table[:, :ncol].astype(np.int64)).cuda()
    pages = pool[idx]                                          # [R, ncol, H, P, D]
    R, _, H, _, D = pages.shape
    out = pages.permute(0, 2, 1, 3, 4).reshape(R, H, ncol * P, D)[:, :, :length]
    return out.cpu().numpy().view(np.uint16)


def _write(s, pk, pos, new):
    """The decoder's append on both sides: new[ten] is [R, H, D] uint16."""
    o = pos % pk.P
    pk.write(pos, new)
    if len(new) == 2 and pos % 2 == 0:                         # through the library's append; V from a strided view
        R, H, D = new[0].shape
        k = torch.as_tensor(new[0].view(np.int16)).cuda()
        wide = torch.zeros((R, H * D + 8), dtype=torch.int16, device="cuda")
        wide[:, :H * D] = torch.as_tensor(new[1].view(np.int16)).cuda().view(R, H * D)
        s.append(0, 1, k, wide[:, :H * D].view(R, H, D), pos)
        return
    for ten, x in enumerate(new):
        s.pools[ten].view(torch.int16)[s.slot.long(), :, o, :] = torch.as_tensor(x.view(np.int16)).cuda()


def _compare_tables(s, pk):
    table, refcnt = s.paged_state()
    ncol = (pk.len + pk.P - 1) // pk.P
    assert np.array_equal(table[:, :ncol], pk.table[:, :ncol])
    assert np.all(table[:, ncol:] == -1)
    assert np.array_equal(refcnt, pk.refcnt)
    return table


@pytest.mark.parametrize("B,N,H,S,D,P,len0", [
    (3, 4, 2, 24, 8, 4, 0), (2, 5, 1, 23, 8, 3, 0), (1, 8, 2, 9, 8, 1, 0), (2, 3, 1, 7, 8, 7, 0),
    (2, 64, 1, 40, 8, 16, 0), (1, 100, 1, 12, 8, 5, 0), (1, 1024, 1, 6, 8, 4, 0), (4, 1, 2, 10, 8, 4, 0),
    (3, 6, 2, 40, 16, 8, 21),
])
def test_paged_matches_model_and_dense_gather(B, N, H, S, D, P, len0):
    rng = np.random.default_rng(B * 1000 + N + P)
    R, n_t = B * N, 2
    s = Session(B, N, 64, 64, "f32", 0.5, 1, kv_geom=(n_t, H, S, D), page_len=P, len0=len0)
    pk = PagedKV(B, N, H, S, D, P, n_t)
    dense = [np.zeros((R, H, S, D), np.uint16) for _ in range(n_t)]
    if len0:
        pk.reset(len0)
        for pos in range(len0):                                # history before the test starts: same on both sides
            new = [rng.integers(0, 65536, (R, H, D), dtype=np.uint16) for _ in range(n_t)]
            pk.write(pos, new)
            for d, x in zip(dense, new):
                d[:, :, pos, :] = x
        for ten in range(n_t):
            s.pools[ten].view(torch.int16).copy_(torch.as_tensor(pk.pool[ten].view(np.int16)))
        _compare_tables(s, pk)
    for pos in range(len0, S):
        slot_ref, copies = pk.prepare_append(pos)
        s.prepare_append(pos)
        assert np.array_equal(s.slot.cpu().numpy(), slot_ref), pos
        new = [rng.integers(0, 65536, (R, H, D), dtype=np.uint16) for _ in range(n_t)]
        _write(s, pk, pos, new)
        for d, x in zip(dense, new):
            d[:, :, pos, :] = x
        flag = (rng.random(B) < 0.6).astype(np.int32)
        anc = np.concatenate([b * N + np.sort(rng.integers(0, N, N)) for b in range(B)]).astype(np.int32)
        if pos % 3 == 1:                                       # unsorted ancestors as well
            anc = np.concatenate([b * N + rng.integers(0, N, N) for b in range(B)]).astype(np.int32)
        pk.reindex(anc, flag)
        dense = [orc.gather_kv(d, anc, flag, N, pos + 1, d.copy()) for d in dense]
        s.paged_reindex(0, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        table = _compare_tables(s, pk)
        if pos % 4 == 3 or pos == S - 1:
            for ten in range(n_t):
                assert np.array_equal(_logical(s, ten, table, pos + 1), dense[ten][:, :, :pos + 1]), (pos, ten)
    assert smc.smc_paged_check(s.ctx) == 0
    s.close()


@pytest.mark.parametrize("B,N,H,S,D,P,len0", [
    (3, 4, 2, 24, 8, 4, 0), (2, 5, 1, 23, 8, 3, 0), (1, 8, 2, 9, 8, 1, 0), (2, 3, 1, 7, 8, 7, 0),
    (2, 64, 1, 40, 8, 16, 0), (1, 100, 1, 12, 8, 5, 0), (1, 1024, 1, 6, 8, 4, 0), (4, 1, 2, 10, 8, 4, 0),
    (3, 6, 2, 40, 16, 8, 21), (2, 130, 1, 600, 8, 4, 100),
])
def test_paged_reorder_and_preparation_in_one_launch(B, N, H, S, D, P, len0):
    """smc_paged_reindex_prepare (the table workgroup that finishes a prompt last prepares it for the next position)
    against the CPU model's reindex followed by prepare_append: slots, tables and reference counts bit-exact after
    every step, logical cache content bit-exact against the dense gather.  The last shape has several table workgroups
    per prompt (130 rows, 25 to 37 columns in use, 15 columns per workgroup)."""
    rng = np.random.default_rng(B * 1000 + N + P + 7)
    R, n_t = B * N, 2
    T = min(S, len0 + 48)                                      # positions appended in the test
    s = Session(B, N, 64, 64, "f32", 0.5, 1, kv_geom=(n_t, H, S, D), page_len=P, len0=len0)
    pk = PagedKV(B, N, H, S, D, P, n_t)
    dense = [np.zeros((R, H, S, D), np.uint16) for _ in range(n_t)]
    if len0:
        pk.reset(len0)
        for pos in range(len0):
            new = [rng.integers(0, 65536, (R, H, D), dtype=np.uint16) for _ in range(n_t)]
            pk.write(pos, new)
            for d, x in zip(dense, new):
                d[:, :, pos, :] = x
        for ten in range(n_t):
            s.pools[ten].view(torch.int16).copy_(torch.as_tensor(pk.pool[ten].view(np.int16)))
    slot_ref, _ = pk.prepare_append(len0)
    s.prepare_append(len0)
    for pos in range(len0, T):
        assert np.array_equal(s.slot.cpu().numpy(), slot_ref), pos
        new = [rng.integers(0, 65536, (R, H, D), dtype=np.uint16) for _ in range(n_t)]
        _write(s, pk, pos, new)
        for d, x in zip(dense, new):
            d[:, :, pos, :] = x
        flag = (rng.random(B) < 0.6).astype(np.int32)
        anc = np.concatenate([b * N + np.sort(rng.integers(0, N, N)) for b in range(B)]).astype(np.int32)
        if pos % 3 == 1:
            anc = np.concatenate([b * N + rng.integers(0, N, N) for b in range(B)]).astype(np.int32)
        pk.reindex(anc, flag)
        dense = [orc.gather_kv(d, anc, flag, N, pos + 1, d.copy()) for d in dense]
        if pos + 1 < T:
            slot_ref, _ = pk.prepare_append(pos + 1)
            s.paged_reindex_prepare(0, pos + 1, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        else:
            s.paged_reindex(0, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        table = _compare_tables(s, pk)
        if pos % 4 == 3 or pos == T - 1:
            for ten in range(n_t):
                assert np.array_equal(_logical(s, ten, table, pos + 1), dense[ten][:, :, :pos + 1]), (pos, ten)
    assert smc.smc_paged_check(s.ctx) == 0
    s.close()


def test_paged_argument_errors_and_foreign_ancestors():
    cfg = smc.make_config(2, 4, 64, 8, "f32", 0.5, 0, 2, 1, 10, 8, 2)
    assert smc.smc_paged_workspace_bytes(cfg, 0) == 0 and smc.smc_paged_workspace_bytes(cfg, 11) == 0
    assert smc.smc_paged_pool_bytes(cfg, 4) == 2 * (4 * 3) * 1 * 4 * 8 * 2
    s = Session(2, 4, 64, 8, "f32", 0.5, 0, kv_geom=(2, 1, 10, 8), page_len=4)
    with pytest.raises(smc.SMCError):
        s.prepare_append(1)                                    # positions are appended one by one from 0
    s.prepare_append(0)
    with pytest.raises(smc.SMCError):
        s.prepare_append(0)
    before, _ = s.paged_state()
    anc = torch.tensor([5, 0, 1, 99, 4, 4, -3, 7], dtype=torch.int32).cuda()      # 5, 99, -3: outside their prompt
    s.paged_reindex(0, anc, torch.ones(2, dtype=torch.int32).cuda())
    table, refcnt = s.paged_state()
    assert table[:, 0].tolist() == [before[0, 0], before[0, 0], before[1, 0], before[3, 0],
                                    before[4, 0], before[4, 0], before[6, 0], before[7, 0]]
    assert refcnt.sum() == 8 and smc.smc_paged_check(s.ctx) == 0
    s2 = Session(2, 4, 64, 8, "f32", 0.5, 0, kv_geom=(2, 1, 10, 8))               # dense session: paged calls refuse
    with pytest.raises(smc.SMCError):
        smc.smc_paged_prepare_append(s2.ctx, 0, s2.tokens)
    s.close(); s2.close()


def test_paged_reindex_before_any_append_moves_only_the_state():
    """No position appended yet: the table has no column in use; histories, sums and parities still follow."""
    B, N, T = 3, 5, 8
    R = B * N
    rng = np.random.default_rng(4)
    s = Session(B, N, 64, T, "f32", 0.5, 0, kv_geom=(2, 1, 12, 8), page_len=4, len0=0)
    o = orc.OracleSMC(B, N, 64, T, 0.5, 0, "f32")
    o.hist[:] = rng.integers(0, 64, (R, T)); o.cumlogp[:] = -rng.random(R)
    s.histA.copy_(torch.as_tensor(o.hist)); s.set_state(None, o.cumlogp)
    for it in range(3):
        anc = np.concatenate([b * N + rng.integers(0, N, N) for b in range(B)]).astype(np.int32)
        flag = np.array([1, it % 2, 1], np.int32)
        t = 3 + 2 * it
        o.hist = s.live_hist().copy()                          # columns beyond an earlier t are unspecified after a copy
        s.paged_reindex(t, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        o.reindex(anc, flag, 0, t)
        _, cum, _ = s.state()
        assert np.array_equal(cum, o.cumlogp) and np.array_equal(s.live_hist()[:, :t], o.hist[:, :t])
        table, refcnt = s.paged_state()
        assert np.all(table == -1) and np.all(refcnt == 0)
    s.close()


@pytest.mark.parametrize("B,N,T", [(3, 64, 2048), (2, 100, 4096), (1, 1024, 512), (5, 8, 4096)])
def test_paged_reorder_with_long_histories(B, N, T):
    """Histories long enough that several workgroups share a prompt's copy (the last one to finish flips the
    parities): repeated calls, unsorted ancestors, every prefix length."""
    R = B * N
    rng = np.random.default_rng(B * 7 + N)
    s = Session(B, N, 64, T, "f32", 0.5, 0, kv_geom=(2, 1, 8, 8), page_len=4, len0=5)
    o = orc.OracleSMC(B, N, 64, T, 0.5, 0, "f32", eos_id=-1)
    o.hist[:] = rng.integers(0, 64, (R, T)); o.cumlogp[:] = -rng.random(R)
    s.histA.copy_(torch.as_tensor(o.hist)); s.set_state(None, o.cumlogp)
    par = np.zeros(R, np.int32)
    for t in (T, T - 3, T // 2 + 1, 7, T):
        anc = np.concatenate([b * N + rng.integers(0, N, N) for b in range(B)]).astype(np.int32)
        flag = (rng.random(B) < 0.8).astype(np.int32); flag[0] = 1
        o.hist = s.live_hist().copy()
        s.paged_reindex(t, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        o.reindex(anc, flag, 0, t)
        _, cum, par2 = s.state()
        moved = (anc != np.arange(R)) & (np.repeat(flag, N) != 0)
        assert np.array_equal(par2, par ^ moved.astype(np.int32)); par = par2
        assert np.array_equal(cum, o.cumlogp) and np.array_equal(s.live_hist()[:, :t], o.hist[:, :t]), t
    s.close()


def test_paged_lockstep_with_the_sampler():
    """The whole step with a paged cache: histories, weights and the logical cache follow the oracle's dense run."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=8, N=8, V=4104, layers=1, H=2, S=40, D=64)
    steps, P = 40, 8
    kv0 = [np.zeros((w.R, w.H, w.S, w.D), np.uint16) for _ in range(2)]
    o = orc.OracleSMC(w.B, w.N, w.V, steps, w.kappa, 0, w.dtype, kv=kv0)
    s = Session(w.B, w.N, w.V, steps, w.dtype, w.kappa, 0, kv_geom=(2, w.H, w.S, w.D), page_len=P)
    rng = np.random.default_rng(5)
    n_res = 0
    for t in range(1, steps + 1):
        pos = t - 1                                            # the decoder appends position t-1, then emits logits
        s.prepare_append(pos)
        new = [rng.integers(0, 65536, (w.R, w.H, w.D), dtype=np.uint16) for _ in range(2)]
        for ten in range(2):
            o.kv[ten][:, :, pos, :] = new[ten]
            s.pools[ten].view(torch.int16)[s.slot.long(), :, pos % P, :] = torch.as_tensor(new[ten].view(np.int16)).cuda()
        x = synth.logits_numpy(w, t, 0)
        want = o.step(x, t, w.alpha, w.alpha)
        s.step(to_device_logits(x, w.dtype), t, w.alpha, w.alpha)
        assert np.array_equal(s.tokens.cpu().numpy(), want["tokens"]) or (want["gap"] < 1e-6).any()
        anc_ref, flag_ref, _ = o.resample(t)
        s.resample(t)
        assert np.array_equal(s.resampled.cpu().numpy(), flag_ref) and np.array_equal(s.anc.cpu().numpy(), anc_ref), t
        o.reindex(anc_ref, flag_ref, t, t)
        s.paged_reindex(t)
        n_res += int(flag_ref.sum())
        logW, cum, _ = s.state()
        assert np.abs(logW - o.logW).max() < 1e-4 and np.abs(cum - o.cumlogp).max() < 1e-4
        if t % 8 == 0:
            assert np.array_equal(s.live_hist()[:, :t], o.hist[:, :t])
            table, _ = s.paged_state()
            for ten in range(2):
                assert np.array_equal(_logical(s, ten, table, t), o.kv[ten][:, :, :t]), (t, ten)
    assert n_res > 10 and smc.smc_paged_check(s.ctx) == 0
    s.close()
