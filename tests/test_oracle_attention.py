"""Pins of the decode-attention oracle: closed forms and an independent library routine (torch CPU SDPA in fp64)."""
import numpy as np
import torch

from oracle.attention import bf16_bits_to_f64, decode_attention
from paper_2602_10273_amd import synth


def _bits(x):
    return synth.f32_to_bf16_bits(np.ascontiguousarray(x, np.float32))


def test_matches_torch_sdpa_in_fp64():
    rng = np.random.default_rng(0)
    for (R, Hq, Hkv, S, D, length) in [(3, 4, 2, 9, 8, 9), (2, 7, 1, 33, 16, 20), (2, 8, 8, 5, 64, 1), (1, 28, 4, 40, 128, 37)]:
        q = _bits(rng.standard_normal((R, Hq, D))); k = _bits(rng.standard_normal((R, Hkv, S, D))); v = _bits(rng.standard_normal((R, Hkv, S, D)))
        scale = 1.0 / np.sqrt(D)
        got = decode_attention(q, k, v, length, scale)
        G = Hq // Hkv
        tq = torch.as_tensor(bf16_bits_to_f64(q)).unsqueeze(2)                            # [R, Hq, 1, D]
        tk = torch.as_tensor(bf16_bits_to_f64(k[:, :, :length])).repeat_interleave(G, dim=1)
        tv = torch.as_tensor(bf16_bits_to_f64(v[:, :, :length])).repeat_interleave(G, dim=1)
        want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale).squeeze(2).numpy()
        assert np.abs(got - want).max() < 1e-12


def test_closed_forms():
    rng = np.random.default_rng(1)
    R, Hq, Hkv, S, D = 2, 4, 2, 12, 8
    v = _bits(rng.standard_normal((R, Hkv, S, D)))
    # equal keys: uniform weights, the output is the mean of the values over the valid positions only
    k = _bits(np.ones((R, Hkv, S, D)))
    q = _bits(rng.standard_normal((R, Hq, D)))
    out = decode_attention(q, k, v, 7, 0.3)
    mean = bf16_bits_to_f64(v)[:, :, :7].mean(axis=2)
    assert np.abs(out - np.repeat(mean, 2, axis=1)).max() < 1e-12
    # zero query: the same; one position: that position's value; head h*G+g reads KV head h
    out = decode_attention(_bits(np.zeros((R, Hq, D))), _bits(rng.standard_normal((R, Hkv, S, D))), v, 7, 1.0)
    assert np.abs(out - np.repeat(mean, 2, axis=1)).max() < 1e-12
    out = decode_attention(q, _bits(rng.standard_normal((R, Hkv, S, D))), v, 1, 1.0)
    assert np.array_equal(out, np.repeat(bf16_bits_to_f64(v)[:, :, 0], 2, axis=1))
    # a key far larger along q than all others takes all the mass (one-hot limit)
    kk = rng.standard_normal((R, Hkv, S, D)) * 0.01
    qq = np.zeros((R, Hq, D)); qq[..., 0] = 8.0
    kk[:, :, 5, 0] = 16.0
    out = decode_attention(_bits(qq), _bits(kk), v, S, 1.0)
    assert np.abs(out - np.repeat(bf16_bits_to_f64(v)[:, :, 5], 2, axis=1)).max() < 1e-9
    # shifting every score of a row by a constant (a key component common to all positions) changes nothing
    k1 = rng.standard_normal((R, Hkv, S, D)); k1[..., 3] = rng.integers(-8, 8, (R, Hkv, S)) / 8.0    # exact in bf16, also + 4
    k2 = k1.copy(); k2[..., 3] += 4.0
    q3 = rng.standard_normal((R, Hq, D))
    k1 = bf16_bits_to_f64(_bits(k1)); k2[..., :3] = k1[..., :3]; k2[..., 4:] = k1[..., 4:]
    a = decode_attention(_bits(q3), _bits(k1), v, S, 0.5); b = decode_attention(_bits(q3), _bits(k2), v, S, 0.5)
    assert np.abs(a - b).max() < 1e-9
