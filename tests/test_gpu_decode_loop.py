"""End-to-end decode loop on a small random-init decoder: Power-SMC with the double-buffered cache and with the paged
cache must generate the same tokens, weights and logical caches (the two layouts hold the same logical content, the
attention kernel reads both in place), and the attention output inside the loop must match the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

import bench_decode
from oracle.attention import decode_attention
from paper_2602_10273_amd.harness import Session

pytestmark = pytest.mark.gpu


def _loop(model, paged, B, N, S, P, steps, alpha, kappa, seed, probe):
    R = B * N
    s = Session(B, N, model.V, 32, "bf16", kappa, seed, kv_geom=(2 * model.L, model.Hkv, S, model.D),
                page_len=P if paged else 0, len0=0)
    parity = None if paged else s.parity_view()
    scale = 1.0 / math.sqrt(model.D)
    state = dict(pos=0)

    def write_kv(layer, k, v):
        pos = state["pos"]
        if layer % 2 == 0:                                     # the library's append; the other layers store by hand
            s.append(2 * layer, 2 * layer + 1, k, v, pos)
            return
        for ten, x in ((2 * layer, k), (2 * layer + 1, v)):
            if paged:
                s.pools[ten][s.slot.long(), :, pos % P, :] = x
            else:
                live_b = (parity != 0).view(R, 1, 1)
                s.kvA[ten][:, :, pos, :] = torch.where(live_b, s.kvA[ten][:, :, pos, :], x)
                s.kvB[ten][:, :, pos, :] = torch.where(live_b, x, s.kvB[ten][:, :, pos, :])

    def attend(layer, q, length):
        out = s.attention(2 * layer, 2 * layer + 1, q, length, scale)
        if probe is not None and layer == 1 and length in (1, 9, steps):
            probe.append((length, q.view(torch.int16).cpu().numpy().view(np.uint16), _dense(s, paged, 2, length),
                          _dense(s, paged, 3, length), out.cpu().numpy()))
        return out

    tokens = torch.zeros(R, dtype=torch.int64, device="cuda")
    hist, n_res = [], 0
    for t in range(1, steps + 1):
        if paged:
            s.prepare_append(state["pos"])
        logits = model.step(tokens, state["pos"], write_kv, attend)
        s.step(logits, t, alpha, alpha, -1.0)
        s.resample(t)
        n_res += int(s.resampled.sum().item())
        if paged:
            s.paged_reindex(t)
        else:
            s.reindex(state["pos"] + 1, t)
        tokens = s.tokens.long()
        state["pos"] += 1
        hist.append(s.live_hist()[:, :t].copy())
    logW, cum, _ = s.state()
    caches = [_dense(s, paged, ten, steps) for ten in range(2 * model.L)]
    s.close()
    return hist[-1], logW, cum, caches, n_res


def _dense(s, paged, ten, length):
    """uint16 [R, Hkv, length, D]: the logical cache of tensor `ten`."""
    if not paged:
        return s.live_kv(ten)[:, :, :length]
    table, _ = s.paged_state()
    P = s.page_len
    ncol = (length + P - 1) // P
    idx = torch.as_tensor(table[:, :ncol].astype(np.int64)).cuda()
    pages = s.pools[ten].view(torch.int16)[idx]
    R, _, H, _, D = pages.shape
    return pages.permute(0, 2, 1, 3, 4).reshape(R, H, ncol * P, D)[:, :, :length].cpu().numpy().view(np.uint16)


def test_dense_and_paged_decode_loops_agree_and_attention_matches_the_oracle():
    model = bench_decode.RandomInitDecoder(bench_decode.SHAPES["tiny"], "cuda", 0)
    model.head *= 12.0                                          # logits spread enough for the weights to degenerate
    B, N, S, P, steps = 3, 8, 24, 4, 20
    probe = []
    h_d, w_d, c_d, kv_d, n_d = _loop(model, False, B, N, S, P, steps, 4.0, 0.9, 5, probe)
    h_p, w_p, c_p, kv_p, n_p = _loop(model, True, B, N, S, P, steps, 4.0, 0.9, 5, None)
    assert n_d > 3 and n_d == n_p                               # resampling happened, and at the same steps
    assert np.array_equal(h_d, h_p)
    assert np.array_equal(w_d, w_p) and np.array_equal(c_d, c_p)
    for a, b in zip(kv_d, kv_p):
        assert np.array_equal(a, b)
    assert len(probe) == 3
    for length, qb, kb, vb, out in probe:
        want = decode_attention(qb, kb, vb, length, 1.0 / math.sqrt(model.D))
        assert np.abs(out - want).max() < 1e-4, length
