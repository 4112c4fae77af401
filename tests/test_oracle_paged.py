"""Pins of the paged-KV oracle: its logical content must equal the dense row gather (the plain definition of the
reorder step, Alg. 1 / App. C) after any sequence of appends and resampling events."""
import numpy as np
import pytest

from oracle import reference as orc
from oracle.paged import PagedKV


def _check_invariants(pk):
    ncol = (pk.len + pk.P - 1) // pk.P
    cnt = np.zeros_like(pk.refcnt)
    for r in range(pk.R):
        b = r // pk.N
        for j in range(pk.M):
            p = pk.table[r, j]
            if j < ncol:
                assert b * pk.Q <= p < (b + 1) * pk.Q          # a prompt only references its own pages
                cnt[p] += 1
    assert np.array_equal(cnt, pk.refcnt)                      # reference counts are the number of references


def _run(B, N, H, S, D, P, n_tensors, seed, p_resample=0.5, worst=False):
    rng = np.random.default_rng(seed)
    R = B * N
    pk = PagedKV(B, N, H, S, D, P, n_tensors)
    dense = [np.zeros((R, H, S, D), np.uint16) for _ in range(n_tensors)]
    for pos in range(S):
        slot, copies = pk.prepare_append(pos)
        j, o = divmod(pos, P)
        assert len(set(slot.tolist())) == R                    # every row owns the page it is about to write
        assert all(pk.refcnt[s] == 1 for s in slot)
        if o == 0:
            assert copies == []
        new = [rng.integers(0, 65536, (R, H, D), dtype=np.uint16) for _ in range(n_tensors)]
        pk.write(pos, new)
        for d, x in zip(dense, new):
            d[:, :, pos, :] = x
        _check_invariants(pk)
        # resampling event after the step that produced position pos
        flag = (rng.random(B) < p_resample).astype(np.int32)
        if worst:                                              # permutations: nothing is ever shared or freed
            anc = np.concatenate([b * N + rng.permutation(N) for b in range(B)]).astype(np.int32)
        else:
            anc = np.concatenate([b * N + np.sort(rng.integers(0, N, N)) for b in range(B)]).astype(np.int32)
        pk.reindex(anc, flag)
        dense = [orc.gather_kv(d, anc, flag, N, pos + 1, d.copy()) for d in dense]
        _check_invariants(pk)
        for ten in range(n_tensors):
            assert np.array_equal(pk.logical(ten), dense[ten][:, :, :pos + 1, :]), (pos, ten)
    return pk


@pytest.mark.parametrize("B,N,H,S,D,P", [(2, 4, 2, 12, 4, 4), (3, 5, 1, 11, 2, 3), (1, 8, 2, 9, 2, 1),
                                         (2, 3, 1, 7, 2, 16), (1, 16, 1, 20, 2, 5)])
def test_paged_cache_equals_dense_gather(B, N, H, S, D, P):
    for seed in range(3):
        pk = _run(B, N, H, S, D, P, 2, seed)
        # at most N-1 rows of a prompt copy, each the pos % P positions filled so far (none at a page start)
        assert pk.copied_positions <= B * (N - 1) * sum(pos % P for pos in range(S))


def test_pool_never_runs_out_in_the_worst_case():
    _run(2, 6, 1, 12, 2, 4, 1, 0, p_resample=1.0, worst=True)
    _run(2, 6, 1, 12, 2, 4, 1, 1, p_resample=1.0)


def test_hand_worked_example():
    """N=2, P=2, S=4 (M=2, Q=4).  Worked by hand from the rules in the module header."""
    pk = PagedKV(1, 2, 1, 4, 1, 2, 1)
    slot, cp = pk.prepare_append(0)
    assert slot.tolist() == [0, 1] and cp == []
    pk.write(0, [np.array([[[10]], [[20]]], np.uint16)])
    pk.reindex(np.array([1, 1], np.int32), np.array([1], np.int32))            # both rows continue row 1
    assert pk.table[:, 0].tolist() == [1, 1] and pk.refcnt.tolist() == [0, 2, 0, 0]
    slot, cp = pk.prepare_append(1)                                            # row 0 keeps page 1, row 1 takes page 0
    assert slot.tolist() == [1, 0] and cp == [(1, 0)]
    assert pk.pool[0][0, 0, 0, 0] == 20 and pk.refcnt.tolist() == [1, 1, 0, 0]
    pk.write(1, [np.array([[[11]], [[21]]], np.uint16)])
    slot, cp = pk.prepare_append(2)                                            # page start: lowest free pages 2, 3
    assert slot.tolist() == [2, 3] and cp == []
    pk.write(2, [np.array([[[12]], [[22]]], np.uint16)])
    pk.reindex(np.array([0, 0], np.int32), np.array([1], np.int32))
    assert pk.table.tolist() == [[1, 2], [1, 2]] and pk.refcnt.tolist() == [0, 2, 2, 0]
    slot, cp = pk.prepare_append(3)                                            # row 1 copies position 2 into page 0
    assert slot.tolist() == [2, 0] and cp == [(2, 0)]
    assert pk.table.tolist() == [[1, 2], [1, 0]] and pk.refcnt.tolist() == [1, 2, 1, 0]
    pk.write(3, [np.array([[[13]], [[23]]], np.uint16)])
    assert pk.logical(0)[:, 0, :, 0].tolist() == [[20, 11, 12, 13], [20, 11, 12, 23]]


def test_reset_is_append_without_resampling():
    pk = PagedKV(2, 3, 1, 10, 1, 4, 1)
    pk.reset(6)
    want = np.full((6, 3), -1)
    for b in range(2):
        for k in range(3):
            for j in range(2):
                want[b * 3 + k, j] = b * pk.Q + j * 3 + k
    assert np.array_equal(pk.table, want) and pk.len == 6
    _check_invariants(pk)
