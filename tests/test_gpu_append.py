"""smc_kv_append: the new position of every row lands in the buffer (dense) or page (paged) that holds the row, and
nowhere else.  Expected values are plain array assignments."""
import numpy as np
import pytest
import torch

from paper_2602_10273_amd import binding as smc
from paper_2602_10273_amd import synth
from paper_2602_10273_amd.harness import Session

pytestmark = pytest.mark.gpu


def _u16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("H,S,D", [(2, 12, 64), (3, 9, 8), (1, 5, 128)])
def test_dense_append_follows_the_parity_of_each_row(H, S, D):
    B, N = 5, 6
    R = B * N
    w = synth.scaled(synth.WORKLOADS["cfg2"], B=B, N=N, V=64, layers=1, H=H, S=S, D=D)
    rng = np.random.default_rng(H * 100 + D)
    kv = [rng.integers(0, 65536, (R, H, S, D), dtype=np.uint16) for _ in range(3)]
    s = Session(B, N, 64, 8, "f32", 0.5, 0, kv=kv)
    for pos in range(S):
        anc = np.concatenate([b * N + np.sort(rng.integers(0, N, N)) for b in range(B)]).astype(np.int32)
        flag = (rng.random(B) < 0.7).astype(np.int32)
        s.reindex(S, 0, torch.as_tensor(anc).cuda(), torch.as_tensor(flag).cuda())
        _, _, par = s.state()
        before_a = [_u16(t) for t in s.kvA]
        before_b = [_u16(t) for t in s.kvB]
        new = [rng.integers(0, 65536, (R, H, D), dtype=np.uint16) for _ in range(3)]
        dev = [torch.as_tensor(x.view(np.int16)).cuda() for x in new]
        s.append(2, 0, dev[2], dev[0], pos)                    # K = tensor 2, V = tensor 0
        if pos % 2:
            s.append(1, -1, dev[1], None, pos)
        torch.cuda.synchronize()
        for ten in range(3):
            want_a, want_b = before_a[ten].copy(), before_b[ten].copy()
            if ten != 1 or pos % 2:
                want_a[par == 0, :, pos, :] = new[ten][par == 0]
                want_b[par != 0, :, pos, :] = new[ten][par != 0]
            assert np.array_equal(_u16(s.kvA[ten]), want_a) and np.array_equal(_u16(s.kvB[ten]), want_b), (pos, ten)
    assert 0 < par.sum() < R
    s.close()


def test_append_argument_errors():
    B, N, H, S, D = 2, 4, 2, 8, 64
    R = B * N
    s = Session(B, N, 64, 8, "f32", 0.5, 0, kv_geom=(2, H, S, D))
    x = torch.zeros((R, H, D), dtype=torch.bfloat16, device="cuda")
    flat = torch.zeros(R * H * D + 64, dtype=torch.bfloat16, device="cuda")
    for bad in (lambda: smc.smc_kv_append(s.ctx, 2, -1, x, H * D, None, 0, 0),            # tensor out of range
                lambda: smc.smc_kv_append(s.ctx, 0, 0, x, H * D, x, H * D, 0),            # K and V the same tensor
                lambda: smc.smc_kv_append(s.ctx, 0, 1, x, H * D, None, H * D, 0),         # V missing
                lambda: smc.smc_kv_append(s.ctx, 0, -1, x, H * D, None, 0, S),            # position out of range
                lambda: smc.smc_kv_append(s.ctx, 0, -1, x, H * D, None, 0, -1),
                lambda: smc.smc_kv_append(s.ctx, 0, -1, x, H * D - 8, None, 0, 0),        # rows overlap
                lambda: smc.smc_kv_append(s.ctx, 0, -1, x, H * D + 4, None, 0, 0),        # stride not a multiple of 8
                lambda: smc.smc_kv_append(s.ctx, 0, -1, flat.data_ptr() + 2, H * D, None, 0, 0)):   # misaligned
        with pytest.raises(smc.SMCError):
            bad()
    s.close()
    p = Session(B, N, 64, 8, "f32", 0.5, 0, kv_geom=(2, H, S, D), page_len=4, len0=3)
    with pytest.raises(smc.SMCError):
        smc.smc_kv_append(p.ctx, 0, 1, x, H * D, x, H * D, 3)                              # no page for position 3 yet
    p.prepare_append(3)
    smc.smc_kv_append(p.ctx, 0, 1, x, H * D, x, H * D, 3)
    torch.cuda.synchronize()
    p.close()
    n = Session(B, N, 64, 8, "f32", 0.5, 0)                                                # no cache bound
    with pytest.raises(smc.SMCError):
        smc.smc_kv_append(n.ctx, 0, -1, x, H * D, None, 0, 0)
    n.close()
