"""Decode attention over the caches the reorder maintains (double-buffered rows with mixed parities, paged pools with
shared pages) against the fp64 oracle: |out - oracle| <= 1e-4 on N(0,1) data (fp32 accumulation, weights fed to the
matrix cores as bf16 high + low parts)."""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from oracle.attention import decode_attention
from paper_2602_10273_amd import binding as smc
from paper_2602_10273_amd import synth
from paper_2602_10273_amd.harness import Session

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _bits(rng, shape, scale=1.0):
    return synth.f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


def _q_dev(qb):
    return torch.as_tensor(qb.view(np.int16)).cuda().view(torch.bfloat16)


@pytest.mark.parametrize("B,N,Hkv,G,S,D,lengths", [
    (2, 3, 2, 4, 40, 128, (1, 15, 16, 17, 40)), (1, 4, 1, 7, 300, 128, (300, 257)), (2, 2, 4, 1, 64, 64, (64, 33)),
    (1, 2, 2, 16, 48, 64, (48,)), (1, 8, 4, 7, 2048, 128, (2048, 1999)), (3, 2, 8, 4, 100, 128, (100,)),
])
def test_dense_cache_with_mixed_parities(B, N, Hkv, G, S, D, lengths):
    rng = np.random.default_rng(B * 100 + G)
    R, Hq = B * N, Hkv * G
    kv = [_bits(rng, (R, Hkv, S, D)) for _ in range(4)]                       # two layers: K0, V0, K1, V1
    s = Session(B, N, 64, 8, "f32", 0.5, 0, kv=kv, with_hist=False)
    o = orc.OracleSMC(B, N, 64, 8, 0.5, 0, "f32", kv=[k.copy() for k in kv])
    for rnd in range(3):                                                      # rows end up in different buffers
        anc = np.concatenate([b * N + rng.integers(0, N, N) for b in range(B)]).astype(np.int32)
        flag = np.ones(B, np.int32)
        o.reindex(anc, flag, S, 0)
        s.reindex(S, 0, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
    for length in lengths:
        for (kt, vt) in ((0, 1), (2, 3)):
            qb = _bits(rng, (R, Hq, D))
            scale = float(1.0 / np.sqrt(D))
            got = s.attention(kt, vt, _q_dev(qb), length, scale).cpu().numpy()
            want = decode_attention(qb, o.kv[kt], o.kv[vt], length, scale)
            assert np.abs(got - want).max() < TOL, (length, kt, np.abs(got - want).max())
    s.close()


@pytest.mark.parametrize("B,N,Hkv,G,S,D,P", [(2, 4, 2, 7, 70, 128, 16), (1, 6, 4, 2, 45, 64, 5), (2, 3, 1, 8, 33, 128, 1),
                                             (1, 4, 2, 4, 600, 128, 64)])
def test_paged_cache_with_shared_pages(B, N, Hkv, G, S, D, P):
    rng = np.random.default_rng(P)
    R, Hq = B * N, Hkv * G
    s = Session(B, N, 64, 8, "f32", 0.5, 0, kv_geom=(2, Hkv, S, D), with_hist=False, page_len=P)
    dense = [np.zeros((R, Hkv, S, D), np.uint16) for _ in range(2)]
    for pos in range(S):
        s.prepare_append(pos)
        for ten in range(2):
            new = _bits(rng, (R, Hkv, D))
            dense[ten][:, :, pos, :] = new
            s.pools[ten].view(torch.int16)[s.slot.long(), :, pos % P, :] = torch.as_tensor(new.view(np.int16)).cuda()
        if pos % 7 == 3 or pos == S - 2:                                      # resampling: pages become shared
            anc = np.concatenate([b * N + np.sort(rng.integers(0, N, N)) for b in range(B)]).astype(np.int32)
            flag = np.ones(B, np.int32)
            dense = [orc.gather_kv(d, anc, flag, N, pos + 1, d.copy()) for d in dense]
            s.paged_reindex(0, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        if pos in (0, S // 2, S - 1):
            qb = _bits(rng, (R, Hq, D))
            scale = 0.11
            got = s.attention(0, 1, _q_dev(qb), pos + 1, scale).cpu().numpy()
            want = decode_attention(qb, dense[0], dense[1], pos + 1, scale)
            assert np.abs(got - want).max() < TOL, (pos, np.abs(got - want).max())
    with pytest.raises(smc.SMCError):
        s.attention(0, 1, _q_dev(_bits(rng, (R, Hq, D))), S + 1, 0.1)
    s.close()


def test_attention_extremes_and_argument_errors():
    rng = np.random.default_rng(3)
    B, N, Hkv, G, S, D = 1, 2, 2, 4, 64, 128
    R, Hq = B * N, Hkv * G
    k = _bits(rng, (R, Hkv, S, D), 0.05); v = _bits(rng, (R, Hkv, S, D))
    kf = synth.bf16_bits_to_f32(k); kf[:, :, 37, 0] = 40.0; k = synth.f32_to_bf16_bits(kf)      # one dominant position
    s = Session(B, N, 64, 8, "f32", 0.5, 0, kv=[k, v], with_hist=False)
    q = np.zeros((R, Hq, D), np.float32); q[..., 0] = 30.0
    qb = synth.f32_to_bf16_bits(q)
    got = s.attention(0, 1, _q_dev(qb), S, 1.0).cpu().numpy()                # scores up to 1200: no overflow
    want = decode_attention(qb, k, v, S, 1.0)
    assert np.isfinite(got).all() and np.abs(got - want).max() < TOL
    qd = _q_dev(qb)
    for bad in (lambda: s.attention(0, 2, qd, S, 1.0), lambda: s.attention(0, 1, qd, 0, 1.0),
                lambda: s.attention(0, 1, qd, S + 1, 1.0), lambda: s.attention(0, 1, qd, S, -1.0),
                lambda: s.attention(0, 1, qd[:, :3], S, 1.0)):
        with pytest.raises((smc.SMCError, ValueError)):
            bad()
    s.close()


def test_terminated_rows_are_skipped():
    """With an EOS token configured, rows whose particle has terminated are not read: output 0, others unchanged."""
    rng = np.random.default_rng(9)
    B, N, Hkv, G, S, D = 2, 4, 2, 4, 600, 128
    R, Hq = B * N, Hkv * G
    k = _bits(rng, (R, Hkv, S, D)); v = _bits(rng, (R, Hkv, S, D))
    s = Session(B, N, 64, 8, "f32", 0.5, 0, kv=[k, v], with_hist=False, eos_id=5)
    qb = _bits(rng, (R, Hq, D))
    done = np.array([0, 1, 0, 0, 1, 1, 0, 0], np.int32)
    s.set_done(done)
    for length in (S, 40):                                     # several splits / a single one
        got = s.attention(0, 1, _q_dev(qb), length, 0.1).cpu().numpy()
        want = decode_attention(qb, k, v, length, 0.1)
        assert np.all(got[done == 1] == 0.0)
        assert np.abs(got[done == 0] - want[done == 0]).max() < TOL
    s.close()
